// Backward pass: every weight gradient and input gradient of the network as tiled contractions.  Weight gradients
// of the conv layers reduce over B*Ho*Wo positions; they are split into fixed chunks along that axis (split_for),
// each chunk writes its own partial, and wgrad_reduce adds the partials in chunk order -- no atomics, so the
// gradient is bit-identical from run to run.
#include "internal.hpp"
#include "imgconv.hpp"

namespace hts {

// ------------------------------------------------------------------------------------------------------------
// conv1 weight gradient for large bf16 batches of small frames with 4, 8, 12 or 16 channels (4x84x84, 16x72x96):
// one workgroup walks a share of the observations.  For each one the sample's 32-channel output gradient [P1][32] is
// copied into LDS, and, four input channels at a time, the frame is converted to bf16 ONCE into an LDS image
// [(c,y)][W]; wavefront t then owns the 32 weight columns (c = 4*group + t/2, u = 4(t%2)..+3, v = 0..7) and adds
//   D[n][(c,u,v)] += sum_m dy[m][n] * image[c][4oy+u][4ox+v]
// over the sample's positions, 16 per matrix instruction.  Both operands have the reduction (the position) as their
// slow index in LDS; the transposing LDS read hands each lane the 8 positions of its row / column -- for the image
// with a per-lane address, so the im2col matrix is never materialised.  (The tile kernel converts every pixel four
// times and fetches it in 8-byte pieces: it is bound by that.)  Positions are padded to a multiple of 16 with zero
// gradient rows.  The bias column is the column sums of the gradient, taken by the copying threads, against the
// constant 255 (the reduction scales every conv1 column by 1/255).  Partials part[workgroup][32][64C+1], combined in workgroup order by the reduction kernel.
// ------------------------------------------------------------------------------------------------------------
// Column sums of a sample share's gradient rows from the per-thread sums bl[NTH][8] (thread t holds columns
// 8 (t % 4) .. + 7): column tid (< 32) is returned to thread tid.  Four groups of 32 threads each add a quarter of a
// column's NTH/4 terms in thread order (their loads batched: one thread walking all of them alone paid an LDS round trip
// per term, 10 us at the end of a 20 us kernel), and the four sums are added in order.  Fixed shape: deterministic.
// Every thread of the workgroup (at least 128) must call it; it contains a barrier; bl[NTH*8 .. +127] is used too.
template <int NTH> __device__ __forceinline__ float bias_column_sum(float *bl, int tid)
{
    constexpr int TERMS = NTH / 4, QUARTER = TERMS / 4;
    static_assert(TERMS % 4 == 0 && QUARTER % 8 == 0, "term counts");
    float *cs = bl + NTH * 8;
    if (tid < 128) {
        const int col = tid & 31, chunk = tid >> 5;
        const float *src = bl + ((col >> 3) + 4 * chunk * QUARTER) * 8 + (col & 7);
        float t = 0.0f;
        for (int k0 = 0; k0 < QUARTER; k0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = src[(k0 + u) * 32];
#pragma unroll
            for (int u = 0; u < 8; ++u) t += v[u];
        }
        cs[chunk * 32 + col] = t;
    }
    __syncthreads();
    return tid < 32 ? ((cs[tid] + cs[32 + tid]) + cs[64 + tid]) + cs[96 + tid] : 0.0f;
}

struct Conv1WgImgArgs {
    const uint8_t *obs;
    const int32_t *index;
    const bf16_t *dy;       // [B][P1][32]
    float *part;
    int B, H, W, W1, P1, N; // N = 64*C + 1
    FastDiv dW1;
};
constexpr int C1WG_THREADS = 512;          // 8 wavefronts = the 8 column tiles of four input channels
constexpr int C1WG_NV = 4;                 // 16-byte vectors of a four-channel slab per thread (a slab of at most 32 KB)
constexpr int C1WG_DYV = 4;                // 16-byte vectors of the sample's output gradient per thread

// PADDED: P1 is not a multiple of 16 (the last step has padding positions)
template <int NG, bool PADDED> __global__ __launch_bounds__(C1WG_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void conv1_wgrad_image_kernel(const Conv1WgImgArgs a)
{
    constexpr int C = 4 * NG;
    extern __shared__ __attribute__((aligned(16))) unsigned char c1w_smem[];
    bf16_t *img = reinterpret_cast<bf16_t *>(c1w_smem);           // one channel group: [(c,y)][W]
    const int rows = 4 * a.H, Wp = a.W;
    bf16_t *dyl = img + ((rows * Wp + 7) & ~7);                   // [P1 padded to 16][32]
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int kg = lane >> 5, g1 = (lane >> 4) & 1, jj = (lane & 15) >> 2, q = lane & 3;
    // frame -> image: the slab's 4*H*W bytes are contiguous in memory and its image is contiguous in LDS (pitch = W),
    // so the copy is linear: 16 pixels per 16-byte load, converted once, two 16-byte LDS stores
    const int nv = (rows * Wp) >> 4;                              // 16-byte vectors of a slab
    const int nvec = a.P1 * 4;                                    // 16-byte vectors in one sample's [P1][32]
    const int nks = (a.P1 + 15) >> 4;                             // matrix-instruction steps per sample and group
    uint4 raw[C1WG_NV];
    bf16x8 dyr[C1WG_DYV];
    auto fetch_image = [&](int b, int cg) {
        const uint8_t *src = a.obs + ((long long)(a.index ? a.index[b] : b) * C + 4 * cg) * a.H * a.W;
#pragma unroll
        for (int i = 0; i < C1WG_NV; ++i) raw[i] = *reinterpret_cast<const uint4 *>(src + 16 * min(tid + i * C1WG_THREADS, nv - 1));
    };
    auto fetch_dy = [&](int b) {
        const bf16_t *dsrc = a.dy + (long long)b * a.P1 * 32;
#pragma unroll
        for (int i = 0; i < C1WG_DYV; ++i) {
            const int v = tid + i * C1WG_THREADS;
            if (v < nvec) dyr[i] = *reinterpret_cast<const bf16x8 *>(dsrc + v * 8);
        }
    };
    // this lane's part of the operand addresses.  Transposing read: lane 4j+q of a 16-lane group points at entries
    // 4q..4q+3 (of the group's 16 rows / columns) at reduction index j and receives the four reduction indices of
    // entry (lane % 16); groups 0,1 hold entries 0-15 and 16-31 at reduction 0-7 (two reads), groups 2,3 at 8-15.
    const int col0 = 16 * g1 + 4 * q;                             // first of the four columns this lane points at
    const bf16_t *a_lane = dyl + (8 * kg + jj) * 32 + col0;
    typedef i16x4 __attribute__((address_space(3))) *lds_ptr;
    auto tr4 = [](const bf16_t *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p)); };
    auto join = [](const i16x4 lo, const i16x4 hi) {
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        const i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };
    f32x16 acc[NG];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
#pragma unroll
        for (int cg = 0; cg < NG; ++cg) acc[cg][r] = 0.0f;
    }
    // Bias column: the column sums of the gradient rows, taken by the threads that copy them into LDS (columns
    // 8 (tid % 4) .. + 7 each) and added in thread order at the end.  (As products against a constant in wavefront 0,
    // that wavefront issued twice the matrix instructions of the others, who waited for it at every barrier.)
    float bsum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bsum[e] = 0.0f;
    // Positions m = 16 ks + 8 kg + jj (first read) and m + 4 (second read) of step ks: where a lane's two image reads of a
    // step start is the same for every sample and channel group, so it is tabulated once (LDS addresses, wave-independent
    // part; one 8-byte entry per step and lane, one row more than there are steps so that the read-ahead needs no check).
    // Walking the positions in registers cost about twenty vector instructions per matrix instruction, and these kernels
    // are bound by exactly that.  The padding positions of the last step (their gradient rows are zero) read position 0.
    typedef __attribute__((address_space(3))) unsigned char *lds_bytes;
    uint2 *tab = reinterpret_cast<uint2 *>(dyl + nks * 16 * 32);
    for (int e = tid; e < (nks + 1) * 64; e += C1WG_THREADS) {
        const int ks = e >> 6 < nks ? e >> 6 : 0, l = e & 63;
        const int lkg = l >> 5, lg1 = (l >> 4) & 1, ljj = (l & 15) >> 2, lq = l & 3, lcol0 = 16 * lg1 + 4 * lq;
        int ma = 16 * ks + 8 * lkg + ljj, mb = ma + 4;
        ma = (PADDED && ma >= a.P1) ? 0 : ma; mb = (PADDED && mb >= a.P1) ? 0 : mb;
        const int oya = a.dW1.div(ma), oxa = ma - oya * a.W1, oyb = a.dW1.div(mb), oxb = mb - oyb * a.W1;
        const int lane_part = (lcol0 >> 3) * Wp + (lcol0 & 7);
        const uint32_t base = (uint32_t)(uintptr_t)(lds_bytes)(unsigned char *)img;
        tab[e] = make_uint2(base + 2u * (uint32_t)(lane_part + 4 * oya * Wp + 4 * oxa),
                            base + 2u * (uint32_t)(lane_part + 4 * oyb * Wp + 4 * oxb));
    }
    const uint32_t wave_img = 2u * (uint32_t)(((w >> 1) * a.H + 4 * (w & 1)) * Wp);      // this wavefront's channel and row half, in bytes
    // zero rows behind the sample's gradient (written once: the copies below never touch them)
    for (int v = nvec + tid; v < nks * 64; v += C1WG_THREADS) *reinterpret_cast<bf16x8 *>(dyl + v * 8) = zero_vec<bf16_t, 8>();

    if ((int)blockIdx.x < a.B) { fetch_image(blockIdx.x, 0); fetch_dy(blockIdx.x); }
    for (int b = blockIdx.x; b < a.B; b += gridDim.x) {
#pragma unroll
        for (int cg = 0; cg < NG; ++cg) {
            if (cg > 0) __syncthreads();      // the previous group's image has been read
#pragma unroll
            for (int i = 0; i < C1WG_NV; ++i) {
                const int v = tid + i * C1WG_THREADS;
                if (v >= nv) continue;
                const uint32_t x[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
                bf16x8 lo, hi;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    lo[e] = from_f32<bf16_t>((float)((x[0] >> (8 * e)) & 0xFFu));
                    lo[4 + e] = from_f32<bf16_t>((float)((x[1] >> (8 * e)) & 0xFFu));
                    hi[e] = from_f32<bf16_t>((float)((x[2] >> (8 * e)) & 0xFFu));
                    hi[4 + e] = from_f32<bf16_t>((float)((x[3] >> (8 * e)) & 0xFFu));
                }
                *reinterpret_cast<bf16x8 *>(img + v * 16) = lo;
                *reinterpret_cast<bf16x8 *>(img + v * 16 + 8) = hi;
            }
            if (cg == 0) {
#pragma unroll
                for (int i = 0; i < C1WG_DYV; ++i) {
                    const int v = tid + i * C1WG_THREADS;
                    if (v < nvec) {
                        *reinterpret_cast<bf16x8 *>(dyl + v * 8) = dyr[i];
#pragma unroll
                        for (int e = 0; e < 8; ++e) bsum[e] += to_f32(dyr[i][e]);
                    }
                }
            }
            __syncthreads();
            // the next image (and, with it, the next sample's gradient) travels while this one is multiplied
            if (cg + 1 < NG) fetch_image(b, cg + 1);
            else if (b + (int)gridDim.x < a.B) { fetch_image(b + gridDim.x, 0); fetch_dy(b + gridDim.x); }

            const bf16_t *ap = a_lane;
            const uint2 *tp = tab + lane;
            // Software pipeline: the four reads of step k+1 are issued before the matrix instruction of step k (the
            // transposing reads are not moved by the compiler), and the table entry of step k+2 before them.  Whole
            // groups of 5 steps are written out.
            auto walk = [&]() {
                i16x4 ra0, ra1, rb0, rb1;
                uint2 tn = tp[0];
                auto read = [&](int ks) {                      // the operands of step ks; tn holds its table entry
                    const uint2 t = tn;
                    tn = tp[(ks + 1) * 64];
                    ra0 = tr4(ap); ra1 = tr4(ap + 4 * 32);
                    rb0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)(t.x + wave_img));
                    rb1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)(t.y + wave_img));
                    ap += 16 * 32;
                };
                auto mult = [&](const bf16x8 av, const bf16x8 bv) {
                    acc[cg] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[cg], 0, 0, 0);
                };
                read(0);
                int ks = 0;
                for (; ks + 5 < nks; ks += 5) {                // steps ks..ks+4; step ks+5 exists and is read in the last turn
#pragma unroll
                    for (int u = 0; u < 5; ++u) {
                        const bf16x8 av = join(ra0, ra1), bv = join(rb0, rb1);
                        read(ks + u + 1);
                        __builtin_amdgcn_sched_barrier(0);     // keep the reads of the next step ahead of this step's product
                        mult(av, bv);
                    }
                }
                for (; ks < nks; ++ks) {
                    const bf16x8 av = join(ra0, ra1), bv = join(rb0, rb1);
                    if (ks + 1 < nks) read(ks + 1);
                    mult(av, bv);
                }
            };
            walk();
        }
        __syncthreads();          // image and gradient are overwritten by the next sample
    }
    // accumulator register r of lane l is D[n = 8(r/4) + 4(l/32) + r%4][column l%32]
#pragma unroll
    for (int cg = 0; cg < NG; ++cg) {
        float *dst = a.part + (long long)blockIdx.x * 32 * a.N + cg * 256 + w * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) dst[(long long)(8 * (r / 4) + 4 * kg + (r % 4)) * a.N] = acc[cg][r];
    }
    // (every wavefront has left the image: the threads' column sums take its place)
    float *bl = reinterpret_cast<float *>(c1w_smem);
#pragma unroll
    for (int e = 0; e < 8; ++e) bl[tid * 8 + e] = bsum[e];
    __syncthreads();
    const float bias = bias_column_sum<C1WG_THREADS>(bl, tid);
    if (tid < 32) a.part[(long long)blockIdx.x * 32 * a.N + (long long)tid * a.N + 64 * C] = 255.0f * bias;
}

static size_t conv1_wgrad_image_lds(const Geom &g)
{
    const size_t nks = (size_t)((g.P1 + 15) / 16);
    return (((size_t)4 * g.H * g.W + 7) & ~(size_t)7) * 2 + nks * 16 * 64 + (nks + 1) * 64 * 8;     // image, gradient rows, address table
}

// true if the frame shape and pointers fit conv1_wgrad_image_kernel
static bool conv1_wgrad_image_fits(const Geom &g, const uint8_t *obs)
{
    if ((g.C != 4 && g.C != 8 && g.C != 12 && g.C != 16) || ((4 * g.H * g.W) & 15) || (((uintptr_t)obs) & 15u) || g.W1 < 16 || g.P1 < 16)
        return false;
    return 4 * g.H * g.W <= C1WG_NV * C1WG_THREADS * 16 && g.P1 * 4 <= C1WG_DYV * C1WG_THREADS &&
           conv1_wgrad_image_lds(g) <= 160 * 1024;
}

// nz: number of workgroups = number of partials written (at most max_parts)
static hipError_t launch_conv1_wgrad_image(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *part, int max_parts,
                                           int *nz)
{
    const Geom &g = c.g;
    Conv1WgImgArgs a;
    a.obs = obs; a.index = index; a.dy = (const bf16_t *)c.ws.dy1; a.part = part;
    a.B = B; a.H = g.H; a.W = g.W; a.W1 = g.W1; a.P1 = g.P1; a.N = g.K1 + 1;
    a.dW1 = FastDiv::make(g.W1);
    const size_t lds = conv1_wgrad_image_lds(g);
    const bool padded = (g.P1 & 15) != 0;
    void (*kern)(const Conv1WgImgArgs);
    if (padded) kern = g.C == 4 ? conv1_wgrad_image_kernel<1, true> : g.C == 8 ? conv1_wgrad_image_kernel<2, true>
                       : g.C == 12 ? conv1_wgrad_image_kernel<3, true> : conv1_wgrad_image_kernel<4, true>;
    else kern = g.C == 4 ? conv1_wgrad_image_kernel<1, false> : g.C == 8 ? conv1_wgrad_image_kernel<2, false>
                : g.C == 12 ? conv1_wgrad_image_kernel<3, false> : conv1_wgrad_image_kernel<4, false>;
    static std::atomic<bool> attr_set[8] = {};       // raise the dynamic-LDS limit once per instantiation (setting it twice is harmless)
    if (!attr_set[g.C / 4 - 1 + (padded ? 4 : 0)].load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set[g.C / 4 - 1 + (padded ? 4 : 0)].store(true, std::memory_order_release);
    }
    const int grid = B < max_parts ? B : max_parts;
    *nz = grid;
    SiteTimer tm(c, SITE_CONV1_WGRAD);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C1WG_THREADS), lds, c.stream, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------------------
// The same weight gradient for 16-channel frames (16x72x96) with the work split between wavefronts: wavefronts 4-7
// (producers) fetch the next four-channel slab of the frame into registers, convert it into one of TWO LDS images and
// bring in the next sample's output gradient, while wavefronts 0-3 (consumers, one per SIMD next to a producer)
// multiply the current slab -- consumer w owns input channel w of the slab, i.e. two column tiles (rows u = 0..3 and
// 4..7 of the 8x8 window) that share the gradient operand.  In the kernel above every wavefront does both jobs in
// turn, so the compute unit alternates between a conversion phase and a multiply phase (2048 frames: 118 us there).
// One barrier per slab, one more per sample (the gradient rows in LDS are replaced between two samples).
// The bias column (the column sums of the gradient, against the constant 255) is added up by the producer threads as
// they copy the gradient rows into LDS, and their sums are added in thread order at the end.
// ------------------------------------------------------------------------------------------------------------
constexpr int C1WS_THREADS = 512, C1WS_PRODUCERS = 256;
constexpr int C1WS_NP = 7;                 // 16-byte vectors of a slab per producer thread (slab of at most 28 KB)
constexpr int C1WS_DYV = 7;                // 16-byte vectors of a sample's output gradient per producer thread
constexpr int C1WS_DP = 2;                 // steps of operand reads a consumer keeps in flight
constexpr int C1WS_MAX_SAMPLES = 64;       // samples per workgroup (their row indices are read once, into LDS)

// NKS: matrix-instruction steps per sample and slab as a compile-time constant (0: taken from the arguments).  With it
// the consumers' step loop is written out without a branch; in a rolled loop with conditional read-aheads the compiler
// waits for every outstanding LDS read at the top of each step, and a consumer, alone on its SIMD, then sits out an LDS
// round trip per step (115 ticks per matrix instruction, measured with phase stamps).
template <bool PADDED, int NKS> __global__ __launch_bounds__(C1WS_THREADS) void conv1_wgrad_slab_kernel(const Conv1WgImgArgs a)
{
    constexpr int NG = 4, C = 16, PT = C1WS_PRODUCERS, DP = C1WS_DP;
    extern __shared__ __attribute__((aligned(16))) unsigned char c1ws_smem[];
    const int Wp = a.W, slab = 4 * a.H * a.W;                     // bytes of a slab in memory; its bf16 image takes twice that
    const int nks = NKS ? NKS : (a.P1 + 15) >> 4;                 // matrix-instruction steps per sample and slab
    bf16_t *dyl = reinterpret_cast<bf16_t *>(c1ws_smem + 4 * slab);      // [P1 padded to 16][32]
    uint2 *tab = reinterpret_cast<uint2 *>(dyl + nks * 16 * 32);
    int *rowid = reinterpret_cast<int *>(tab + (nks + C1WS_DP) * 64);    // [C1WS_MAX_SAMPLES] rows of this workgroup's samples
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = lane >> 5, g1 = (lane >> 4) & 1, jj = (lane & 15) >> 2, q4 = lane & 3;
    const int nvec = a.P1 * 4;                                    // 16-byte vectors in one sample's [P1][32]
    const int nsamp = (a.B - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int nphase = nsamp * NG;                                // slab p: sample p / NG of this workgroup, channels 4 (p % NG) .. + 3
    typedef __attribute__((address_space(3))) unsigned char *lds_bytes;
    // where a lane's two image reads of a step start (see the kernel above), relative to an image's first byte; DP rows
    // more than there are steps, so that the read-ahead needs no check
    for (int e = tid; e < (nks + C1WS_DP) * 64; e += C1WS_THREADS) {
        const int ks = e >> 6 < nks ? e >> 6 : 0, l = e & 63;
        const int lkg = l >> 5, lg1 = (l >> 4) & 1, ljj = (l & 15) >> 2, lq = l & 3, lcol0 = 16 * lg1 + 4 * lq;
        int ma = 16 * ks + 8 * lkg + ljj, mb = ma + 4;
        ma = (PADDED && ma >= a.P1) ? 0 : ma; mb = (PADDED && mb >= a.P1) ? 0 : mb;
        const int oya = a.dW1.div(ma), oxa = ma - oya * a.W1, oyb = a.dW1.div(mb), oxb = mb - oyb * a.W1;
        const int lane_part = (lcol0 >> 3) * Wp + (lcol0 & 7);
        const uint32_t base = (uint32_t)(uintptr_t)(lds_bytes)c1ws_smem;
        tab[e] = make_uint2(base + 2u * (uint32_t)(lane_part + 4 * oya * Wp + 4 * oxa),
                            base + 2u * (uint32_t)(lane_part + 4 * oyb * Wp + 4 * oxb));
    }
    if (tid < nsamp) { const int b = blockIdx.x + tid * gridDim.x; rowid[tid] = a.index ? a.index[b] : b; }
    // zero rows behind the sample's gradient (written once: the copies below never touch them)
    for (int v = nvec + tid; v < nks * 64; v += C1WS_THREADS) *reinterpret_cast<bf16x8 *>(dyl + v * 8) = zero_vec<bf16_t, 8>();

    f32x16 acc[NG][2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
#pragma unroll
        for (int cg = 0; cg < NG; ++cg) { acc[cg][0][r] = 0.0f; acc[cg][1][r] = 0.0f; }
    }
    float bsum[8];          // producers: column sums of the gradient rows this thread copies (columns 8 (pt % 4) .. + 7): the bias column
#pragma unroll
    for (int e = 0; e < 8; ++e) bsum[e] = 0.0f;
    if (w >= 4) {
        // ---- producers ----
        const int pt = tid - (C1WS_THREADS - PT);
        const int nv = slab >> 4;
        uint4 raw[2][C1WS_NP];
        bf16x8 dyr[C1WS_DYV];
        // A thread's byte offsets inside a slab / a sample's gradient never change; what changes per slab is the same
        // for the whole workgroup and is kept in scalar registers, so a fetch is loads and nothing else (the address
        // arithmetic of seven 64-bit pointers per slab was a fifth of a producer's time beside a busy consumer).
        uint32_t ioff[C1WS_NP], doff[C1WS_DYV];
#pragma unroll
        for (int i = 0; i < C1WS_NP; ++i) ioff[i] = 16u * (uint32_t)min(pt + i * PT, nv - 1);
#pragma unroll
        for (int i = 0; i < C1WS_DYV; ++i) doff[i] = 16u * (uint32_t)min(pt + i * PT, nvec - 1);
        auto fetch_image = [&](int p, uint4 (&r)[C1WS_NP]) {
            const int s = p / NG, cg = p - s * NG;
            const long long row = __builtin_amdgcn_readfirstlane(rowid[s]);
            const uint8_t *src = a.obs + (row * C + 4 * cg) * a.H * a.W;
#pragma unroll
            for (int i = 0; i < C1WS_NP; ++i) r[i] = *reinterpret_cast<const uint4 *>(src + ioff[i]);
        };
        auto fetch_dy = [&](int s) {
            const unsigned char *dsrc = reinterpret_cast<const unsigned char *>(a.dy + (long long)(blockIdx.x + s * gridDim.x) * a.P1 * 32);
#pragma unroll
            for (int i = 0; i < C1WS_DYV; ++i) dyr[i] = *reinterpret_cast<const bf16x8 *>(dsrc + doff[i]);
        };
        auto convert = [&](const uint4 (&r)[C1WS_NP], int buf) {
            unsigned char *dst = c1ws_smem + buf * 2 * slab + 32 * pt;
#pragma unroll
            for (int i = 0; i < C1WS_NP; ++i) {
                if (pt + i * PT >= nv) continue;
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
        };
        auto write_dy = [&]() {
#pragma unroll
            for (int i = 0; i < C1WS_DYV; ++i) {
                const int v = pt + i * PT;
                if (v < nvec) {
                    *reinterpret_cast<bf16x8 *>(dyl + v * 8) = dyr[i];
#pragma unroll
                    for (int e = 0; e < 8; ++e) bsum[e] += to_f32(dyr[i][e]);
                }
            }
        };
        __syncthreads();                                           // the row indices are in LDS
        fetch_image(0, raw[0]);
        fetch_image(1, raw[1]);                                    // (NG > 1: slab 1 always exists)
        fetch_dy(0);
        convert(raw[0], 0);
        write_dy();
        fetch_image(2, raw[0]);
        if (nsamp > 1) fetch_dy(1);
        __syncthreads();
        for (int s = 0; s < nsamp; ++s) {
#pragma unroll
            for (int cg = 0; cg < NG; ++cg) {                     // slab p + 1 sits in register set (cg + 1) % 2
                const int p = s * NG + cg;
                if (p + 1 < nphase) convert(raw[(cg + 1) & 1], (cg + 1) & 1);
                if (p + 3 < nphase) fetch_image(p + 3, raw[(cg + 1) & 1]);
                __syncthreads();
            }
            if (s + 1 < nsamp) {                                  // every consumer has left this sample's gradient rows
                write_dy();
                if (s + 2 < nsamp) fetch_dy(s + 2);
                __syncthreads();
            }
        }
    } else {
        // ---- consumers ----
        // Transposing read: lane 4j+q of a 16-lane group points at entries 4q..4q+3 (of the group's 16 rows / columns) at
        // reduction index j and receives the four reduction indices of entry (lane % 16); groups 0,1 hold entries 0-15
        // and 16-31 at reduction 0-7 (two reads), groups 2,3 at 8-15.
        const int col0 = 16 * g1 + 4 * q4;
        const bf16_t *a_lane = dyl + (8 * kg + jj) * 32 + col0;
        typedef i16x4 __attribute__((address_space(3))) *lds_ptr;
        auto tr4 = [](const bf16_t *p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p)); };
        auto trb = [](uint32_t addr) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(uintptr_t)addr); };
        auto join = [](const i16x4 lo, const i16x4 hi) {
            typedef short i16x8 __attribute__((ext_vector_type(8)));
            const i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            return __builtin_bit_cast(bf16x8, v);
        };
        const uint2 *tp = tab + lane;
        __syncthreads();
        __syncthreads();
        for (int s = 0; s < nsamp; ++s) {
#pragma unroll
            for (int cg = 0; cg < NG; ++cg) {
                // this wavefront's channel of the slab in image (cg & 1), rows u = 0..3 / 4..7 of the window, in bytes
                const uint32_t img0 = (uint32_t)((cg & 1) * 2 * slab + 2 * (w * a.H) * Wp), img1 = img0 + (uint32_t)(2 * 4 * Wp);
                // Software pipeline: the six operand reads of step k+DP are issued before the matrix instructions of step
                // k (a wavefront runs alone on its SIMD here, and one step's products are much shorter than an LDS round
                // trip), and the table entry of step k+2DP with them.  DP operand sets; the loop is written out DP steps at a time.
                struct Ops { i16x4 a0, a1, b0, b1, c0, c1; uint2 tn; };
                Ops o[DP];
                auto read = [&](int ks, Ops &x) {                  // the operands of step ks; x.tn holds its table entry
                    const uint2 t = x.tn;
                    x.tn = tp[(ks + DP) * 64];
                    const bf16_t *ap = a_lane + ks * (16 * 32);
                    x.a0 = tr4(ap); x.a1 = tr4(ap + 4 * 32);
                    x.b0 = trb(t.x + img0); x.b1 = trb(t.y + img0);
                    x.c0 = trb(t.x + img1); x.c1 = trb(t.y + img1);
                };
                auto step = [&](int ks, Ops &x) {
                    const bf16x8 av = join(x.a0, x.a1), bv = join(x.b0, x.b1), cv = join(x.c0, x.c1);
                    if (ks + DP < nks) read(ks + DP, x);
                    __builtin_amdgcn_sched_barrier(0);             // keep those reads ahead of this step's products
                    acc[cg][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[cg][0], 0, 0, 0);
                    acc[cg][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, cv, acc[cg][1], 0, 0, 0);
                };
#pragma unroll
                for (int d = 0; d < DP; ++d) { o[d].tn = tp[d * 64]; if (d < nks) read(d, o[d]); }
                if constexpr (NKS > 0) {
#pragma unroll
                    for (int ks = 0; ks < NKS; ++ks) step(ks, o[ks % DP]);
                } else {
                    int ks = 0;
                    for (; ks + DP <= nks; ks += DP) {
#pragma unroll
                        for (int d = 0; d < DP; ++d) step(ks + d, o[d]);
                    }
#pragma unroll
                    for (int d = 0; d < DP - 1; ++d) if (ks + d < nks) step(ks + d, o[d]);
                }
                __syncthreads();
            }
            if (s + 1 < nsamp) __syncthreads();
        }
        // accumulator register r of lane l is D[n = 8(r/4) + 4(l/32) + r%4][column l%32]
#pragma unroll
        for (int cg = 0; cg < NG; ++cg)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float *dst = a.part + (long long)blockIdx.x * 32 * a.N + cg * 256 + (2 * w + h) * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(long long)(8 * (r / 4) + 4 * kg + (r % 4)) * a.N] = acc[cg][h][r];
            }
    }
    // bias column: the producers' sums, added in thread order; against the constant 255 (the reduction scales every
    // conv1 column by 1/255).  (Every wavefront has left the images: the sums take their place.)
    float *bl = reinterpret_cast<float *>(c1ws_smem);
    if (w >= 4) {
#pragma unroll
        for (int e = 0; e < 8; ++e) bl[(tid - (C1WS_THREADS - PT)) * 8 + e] = bsum[e];
    }
    __syncthreads();
    const float bias = bias_column_sum<PT>(bl, tid);
    if (tid < 32) a.part[(long long)blockIdx.x * 32 * a.N + (long long)tid * a.N + 64 * C] = 255.0f * bias;
}

static size_t conv1_wgrad_slab_lds(const Geom &g)
{
    const size_t nks = (size_t)((g.P1 + 15) / 16);
    return (size_t)16 * g.H * g.W + nks * 16 * 64 + (nks + C1WS_DP) * 64 * 8 + C1WS_MAX_SAMPLES * 4;      // two images, gradient rows, address table, row indices
}

// true if a batch of B samples cut into at most max_parts workgroups leaves each of them no more samples than its index table holds
static bool conv1_wgrad_slab_batch_fits(int B, int max_parts)
{
    const int grid = B < max_parts ? B : max_parts;
    return grid > 0 && (B + grid - 1) / grid <= C1WS_MAX_SAMPLES;
}

// true if the frame shape and pointers fit conv1_wgrad_slab_kernel
static bool conv1_wgrad_slab_fits(const Geom &g, const uint8_t *obs)
{
    return g.C == 16 && !(g.W & 3) && !((g.H * g.W) & 3) && !(((uintptr_t)obs) & 15u) && g.W1 >= 16 && g.P1 >= 16 &&
           4 * g.H * g.W <= C1WS_NP * C1WS_PRODUCERS * 16 && g.P1 * 4 <= C1WS_DYV * C1WS_PRODUCERS &&
           conv1_wgrad_slab_lds(g) <= 160 * 1024;
}

static hipError_t launch_conv1_wgrad_slab(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *part, int max_parts,
                                          int *nz)
{
    const Geom &g = c.g;
    Conv1WgImgArgs a;
    a.obs = obs; a.index = index; a.dy = (const bf16_t *)c.ws.dy1; a.part = part;
    a.B = B; a.H = g.H; a.W = g.W; a.W1 = g.W1; a.P1 = g.P1; a.N = g.K1 + 1;
    a.dW1 = FastDiv::make(g.W1);
    const size_t lds = conv1_wgrad_slab_lds(g);
    const bool padded = (g.P1 & 15) != 0;
    const bool football = g.P1 == 391;               // 16x72x96 frames: 17 x 23 positions, 25 steps
    void (*kern)(const Conv1WgImgArgs) = football ? conv1_wgrad_slab_kernel<true, 25>
                                         : padded ? conv1_wgrad_slab_kernel<true, 0> : conv1_wgrad_slab_kernel<false, 0>;
    static std::atomic<bool> attr_set[3] = {};       // raise the dynamic-LDS limit once per instantiation (setting it twice is harmless)
    const int which = football ? 2 : padded ? 1 : 0;
    if (!attr_set[which].load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set[which].store(true, std::memory_order_release);
    }
    const int grid = B < max_parts ? B : max_parts;
    if ((B + grid - 1) / grid > C1WS_MAX_SAMPLES) return hipErrorInvalidValue;      // (the caller checks conv1_wgrad_slab_batch_fits)
    *nz = grid;
    SiteTimer tm(c, SITE_CONV1_WGRAD);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C1WS_THREADS), lds, c.stream, a);
    return hipGetLastError();
}

template <typename T> static hipError_t backward_t(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *grads)
{
    const Geom &g = c.g;
    hipError_t e;
    // Small minibatches take the wave-per-segment kernels: many more, much shorter dependency chains.
    const bool small = B <= c.small_b;
    const bool atari_grid = g.H1 == 20 && g.W1 == 20;      // 84x84 frames: conv2 sees 20x20, conv3 9x9
    const bool foot_grid = g.H1 == 17 && g.W1 == 23;       // 72x96 frames: conv2 sees 17x23, conv3 7x10
    // groups of 64-row segments for the split weight gradients on that path: at most max_groups partial buffers per
    // layer, at least min_segs segments per group (never more groups than the tile path's split_for allows for the
    // same reduction length, which is what the partial buffers are sized for)
    auto groups_for = [](long long kp, int *spg, int max_groups, int min_segs) {
        const int nseg = (int)((kp + 63) / 64);
        int s = (nseg + max_groups - 1) / max_groups;
        s = ((s + 3) / 4) * 4;
        if (s < min_segs) s = min_segs;
        *spg = s;
        return (nseg + s - 1) / s;
    };
    // heads: pi.w, pi.b, v.w, v.b.  A tiny output and a reduction over the whole minibatch: beyond 512 rows it is cut
    // into groups of 16 segments (one round of the 16 wavefronts) whose partials join the conv layers' reduction.
    int nzh = 0;
    {
        HeadsWgrad p;
        p.M = g.A + 1; p.N = 513; p.K = B; p.klen = B;
        p.dz = c.ws.dz; p.h = c.ws.h; p.g = grads; p.A = g.A; p.part = nullptr;
        p.piw = g.piw; p.pib = g.pib; p.vw = g.vw; p.vb = g.vb;
        const int nseg = (B + 31) / 32;
        int spg = 1 << 30;
        if (nseg > 16) {
            spg = 16 * ((nseg + 16 * HEADS_MAXZ - 1) / (16 * HEADS_MAXZ));      // whole rounds, at most HEADS_MAXZ groups
            nzh = (nseg + spg - 1) / spg;
            p.part = c.ws.heads_part;
        }
        {
            SiteTimer tm(c, SITE_HEADS_WGRAD);        // 16 wavefronts share each tile
            e = launch_wsgemm<HeadsWgrad, 16, 32, false>(p, c.stream, spg);
        }
        if (e != hipSuccess) return e;
    }
    {   // fc.w, fc.b
        FcWgrad<T> p;
        p.M = 512; p.N = g.F + 1; p.K = B; p.klen = B;
        p.dh = (const T *)c.ws.dh; p.a3 = (const T *)c.ws.a3; p.g = grads; p.F = g.F; p.fcw = g.fcw; p.fcb = g.fcb;
        { SiteTimer tm(c, SITE_FC_WGRAD); e = launch_gemm(p, c.stream); }
        if (e != hipSuccess) return e;
    }
    {   // d(conv3 pre-activation)
        FcDgrad<T> p;
        p.M = B; p.N = g.F; p.K = 512; p.klen = 512;
        p.dh = (const T *)c.ws.dh; p.wfcd = (const T *)c.ws.wfcd; p.a3n = (const T *)c.ws.a3n; p.dy3 = (T *)c.ws.dy3;
        {
            SiteTimer tm(c, SITE_FC_DGRAD);
            e = small ? launch_wsgemm<FcDgrad<T>, 4, 64, false>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    // partial buffers of the three conv weight gradients live side by side in ws.part
    const SplitK s3 = split_for((long long)B * g.P3, MAXZ3), s2 = split_for((long long)B * g.P2, MAXZ2),
                 s1 = split_for((long long)B * g.P1, MAXZ1);
    int spg3 = 0, spg2 = 0, spg1 = 0;
    const int nz3 = small ? groups_for((long long)B * g.P3, &spg3, 32, 8) : s3.nz;
    const int nz2 = small ? groups_for((long long)B * g.P2, &spg2, 32, 8) : s2.nz;
    int nz1 = small ? groups_for((long long)B * g.P1, &spg1, 56, 4) : s1.nz;   // long reduction, tiny output
    float *part3 = c.ws.part;
    float *part2 = part3 + (size_t)nz3 * 64 * 577;
    float *part1 = part2 + (size_t)nz2 * 64 * 513;
    {   // conv3.w, conv3.b
        ConvWgrad<T, Layer3> p;
        p.M = 64; p.N = 577; p.K = B * g.P3; p.klen = s3.klen;
        p.dy = (const T *)c.ws.dy3; p.in = (const T *)c.ws.act2; p.part = part3;
        p.Hin = g.H2; p.Win = g.W2; p.Wo = g.W3; p.Po = g.P3;
        p.dPo = FastDiv::make(g.P3); p.dWo = FastDiv::make(g.W3);
        {
            SiteTimer tm(c, SITE_CONV3_WGRAD);
            e = small ? launch_wsgemm<ConvWgrad<T, Layer3>, 4, 64, false>(p, c.stream, spg3) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // d(conv2 pre-activation)
        ConvDgrad<T, Layer3> p;
        p.N = 64; p.K = 576; p.klen = 576;
        p.dy = (const T *)c.ws.dy3; p.wd = (const T *)c.ws.wd3; p.act_in = (const T *)c.ws.act2; p.dy_in = (T *)c.ws.dy2;
        p.Bn = B; p.Hin = g.H2; p.Win = g.W2; p.Ho = g.H3; p.Wo = g.W3;
        p.prepare();
        {
            SiteTimer tm(c, SITE_CONV3_DGRAD);
            if (!small && sizeof(T) == 2 && atari_grid) {      // large bf16 batch, 9x9 input: output gradients resident in LDS
                ImgConvArgs a = {};
                a.in = (const bf16_t *)c.ws.dy3; a.w = (const bf16_t *)c.ws.wd3; a.mask = (const bf16_t *)c.ws.act2;
                a.out = (bf16_t *)c.ws.dy2; a.B = B;
                e = launch_imgconv<ImgDgrad<64, 3, 1, 9, 9, 6>>(a, c.stream);
            } else if (!small && sizeof(T) == 2 && foot_grid) {
                ImgConvArgs a = {};
                a.in = (const bf16_t *)c.ws.dy3; a.w = (const bf16_t *)c.ws.wd3; a.mask = (const bf16_t *)c.ws.act2;
                a.out = (bf16_t *)c.ws.dy2; a.B = B;
                e = launch_imgconv<ImgDgrad<64, 3, 1, 7, 10, 8>>(a, c.stream);
            } else
            // binary32: eight segments of 72 for eight wavefronts, both operands through LDS: a lane that fetches its own
            // weight column touches 32 cache lines per load instruction, and with sixteen wavefronts on a compute unit
            // the L1's address processing was the whole issue phase (24.2 -> 19.3 us at 80 rows).  bfloat16 rows are
            // half as long and the direct form stays faster there (11.6 vs 17.2 us).
            e = small ? launch_wsgemm<ConvDgrad<T, Layer3>, (sizeof(T) == 4 ? 8 : 4), (sizeof(T) == 2 ? 192 : 72), false, (sizeof(T) == 2)>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // conv2.w, conv2.b
        ConvWgrad<T, Layer2> p;
        p.M = 64; p.N = 513; p.K = B * g.P2; p.klen = s2.klen;
        p.dy = (const T *)c.ws.dy2; p.in = (const T *)c.ws.act1; p.part = part2;
        p.Hin = g.H1; p.Win = g.W1; p.Wo = g.W2; p.Po = g.P2;
        p.dPo = FastDiv::make(g.P2); p.dWo = FastDiv::make(g.W2);
        {
            SiteTimer tm(c, SITE_CONV2_WGRAD);
            e = small ? launch_wsgemm<ConvWgrad<T, Layer2>, 4, 64, false>(p, c.stream, spg2) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // d(conv1 pre-activation)
        ConvDgrad<T, Layer2> p;
        p.N = 32; p.K = 256; p.klen = 256;      // four parity classes, 2x2 taps each
        p.dy = (const T *)c.ws.dy2; p.wd = (const T *)c.ws.wd2; p.act_in = (const T *)c.ws.act1; p.dy_in = (T *)c.ws.dy1;
        p.Bn = B; p.Hin = g.H1; p.Win = g.W1; p.Ho = g.H2; p.Wo = g.W2;
        p.prepare();
        {
            SiteTimer tm(c, SITE_CONV2_DGRAD);
            if (!small && sizeof(T) == 2 && atari_grid) {
                ImgConvArgs a = {};
                a.in = (const bf16_t *)c.ws.dy2; a.w = (const bf16_t *)c.ws.wd2; a.mask = (const bf16_t *)c.ws.act1;
                a.out = (bf16_t *)c.ws.dy1; a.B = B;
                e = launch_imgconv<ImgDgrad<32, 4, 2, 20, 20, 4>>(a, c.stream);
            } else if (!small && sizeof(T) == 2 && foot_grid) {
                ImgConvArgs a = {};
                a.in = (const bf16_t *)c.ws.dy2; a.w = (const bf16_t *)c.ws.wd2; a.mask = (const bf16_t *)c.ws.act1;
                a.out = (bf16_t *)c.ws.dy1; a.B = B;
                e = launch_imgconv<ImgDgrad<32, 4, 2, 17, 23, 4>>(a, c.stream);
            } else
            e = small ? launch_wsgemm<ConvDgrad<T, Layer2>, 4, 64, false>(p, c.stream) : launch_gemm(p, c.stream);
        }
        if (e != hipSuccess) return e;
    }
    {   // conv1.w, conv1.b
        auto conv1_wgrad = [&](auto p) {
            p.M = 32; p.N = g.K1 + 1; p.K = B * g.P1; p.klen = s1.klen;
            p.dy = (const T *)c.ws.dy1; p.obs = obs; p.index = index; p.part = part1;
            p.Kc = g.K1; p.C = g.C; p.H = g.H; p.W = g.W; p.W1 = g.W1; p.P1 = g.P1;
            p.dP1 = FastDiv::make(g.P1); p.dW1 = FastDiv::make(g.W1);
            SiteTimer tm(c, SITE_CONV1_WGRAD);
            return small ? launch_wsgemm<decltype(p), 4, 64, false>(p, c.stream, spg1) : launch_gemm(p, c.stream);
        };
        if (!small && sizeof(T) == 2 && B >= c.conv1_slab_rows && conv1_wgrad_slab_fits(g, obs) && conv1_wgrad_slab_batch_fits(B, s1.nz)) e = launch_conv1_wgrad_slab(c, obs, index, B, part1, s1.nz, &nz1);
        else if (!small && sizeof(T) == 2 && conv1_wgrad_image_fits(g, obs)) e = launch_conv1_wgrad_image(c, obs, index, B, part1, s1.nz, &nz1);
        else e = index ? conv1_wgrad(Conv1Wgrad<T, true>{}) : conv1_wgrad(Conv1Wgrad<T, false>{});
        if (e != hipSuccess) return e;
    }
    const long long hstride = (long long)(g.A + 1) * 513;
    const ReduceSpec specs[REDUCE_JOBS] = {
        {part3, nz3, 64, 577, 64, 3, 0, true, 1.0f, g.w3, g.b3},
        {part2, nz2, 64, 513, 32, 4, 0, true, 1.0f, g.w2, g.b2},
        {part1, nz1, 32, g.K1 + 1, g.C, 8, 0, false, 1.0f / 255.0f, g.w1, g.b1},
        {c.ws.heads_part, nzh, g.A, 513, 1, 1, hstride, false, 1.0f, g.piw, g.pib},
        {c.ws.heads_part + (long long)g.A * 513, nzh, 1, 513, 1, 1, hstride, false, 1.0f, g.vw, g.vb}};
    if ((e = launch_wgrad_reduce(c, specs, grads)) != hipSuccess) return e;
    return hipSuccess;
}

hipError_t run_backward(Ctx &c, const uint8_t *obs, const int32_t *index, int B, float *grads)
{
    return c.desc.precision == HTS_PRECISION_BF16 ? backward_t<bf16_t>(c, obs, index, B, grads)
                                                  : backward_t<float>(c, obs, index, B, grads);
}

}  // namespace hts
