// Tiled matrix-multiply core on CDNA4 matrix instructions (gfx950).
//
// Every dense contraction of the network (Nature-CNN of the paper's appendix "Implementation Details") is
// expressed as  D[m][n] = sum_k A(m,k) * B(n,k)  where a small "problem" object supplies the operand gathers
// (implicit im2col, index gather, weight layouts) and the epilogue (bias, ReLU, masks, output layout).
//
// One workgroup = 256 threads = 4 wavefronts of 64 lanes; each wavefront owns a (TM*32) x (TN*32) block of D
// built from 32x32 MFMA accumulators:
//   fp32 : v_mfma_f32_32x32x2_f32   (lane l supplies A[l%32][l/32] and B[l/32][l%32])
//   bf16 : v_mfma_f32_32x32x16_bf16 (lane l supplies 8 consecutive k at k0 = 8*(l/32) for row/col l%32)
// Accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
//
// Operand tiles go global -> registers -> LDS ([row][k], padded) -> MFMA; the global loads of tile i+1 are in
// flight while tile i is multiplied.  blockIdx.y selects a contiguous K range of length p.klen (split-K); the
// problem's store() receives that index so partial sums go to distinct slots and are later combined in a fixed
// order (no atomics anywhere).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#define HTS_HD __host__ __device__ __forceinline__

namespace hts {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct OperandTraits;
template <> struct OperandTraits<float> {
    static constexpr int KINST = 2;   // k consumed per MFMA
    static constexpr int PAD = 1;     // LDS row padding (elements)
    static constexpr int VEC = 4;     // elements per 16-byte global access
};
template <> struct OperandTraits<bf16_t> {
    static constexpr int KINST = 16;
    static constexpr int PAD = 8;
    static constexpr int VEC = 8;
};

HTS_HD float to_f32(float x) { return x; }
HTS_HD float to_f32(bf16_t x) { return (float)x; }
template <typename T> HTS_HD T from_f32(float x);
template <> HTS_HD float from_f32<float>(float x) { return x; }
template <> HTS_HD bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }   // round to nearest even

// 16-byte (or shorter) contiguous loads returning floats
HTS_HD void load_vec(const float *p, float (&v)[4])
{
    const f32x4 t = *reinterpret_cast<const f32x4 *>(p);
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
HTS_HD void load_vec(const bf16_t *p, float (&v)[8])
{
    const bf16x8 t = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
}
HTS_HD void load_vec(const float *p, float (&v)[8])
{
    const f32x4 t0 = *reinterpret_cast<const f32x4 *>(p);
    const f32x4 t1 = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = t0[i]; v[4 + i] = t1[i]; }
}
HTS_HD void load_vec(const bf16_t *p, float (&v)[4])
{
    const bf16x4 t = *reinterpret_cast<const bf16x4 *>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (float)t[i];
}
HTS_HD void load_vec(const float *p, float (&v)[1]) { v[0] = *p; }
template <int V> HTS_HD void zero_vec(float (&v)[V])
{
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] = 0.0f;
}

// Optional segmented accumulation: a problem that defines `static constexpr int SEG` (a multiple of BK) gets
//   D = (((s_0 + s_1) + s_2) + ...),  s_i = MFMA-accumulated sum over k in [i*SEG, (i+1)*SEG)
// instead of one long accumulation chain.  The wave-per-segment kernel of wsgemm.hpp computes the s_i in parallel
// and adds them in the same order, so both kernels return identical bits for the same problem.
template <class P, class = void> struct SegOf { static constexpr int value = 0; };
template <class P> struct SegOf<P, std::void_t<decltype(P::SEG)>> { static constexpr int value = P::SEG; };

// Optional batching: a problem with `int batches() const`, `int max_m() const` and `void set_batch(int)` is launched
// with gridDim.z = batches(); each z works on its own sub-problem (own M, own gathers) selected by set_batch.
template <class P, class = void> struct HasBatch : std::false_type {};
template <class P> struct HasBatch<P, std::void_t<decltype(std::declval<const P &>().batches())>> : std::true_type {};
template <class P> inline int grid_rows(const P &p)
{
    if constexpr (HasBatch<P>::value) return p.max_m(); else return p.M;
}
template <class P> inline int grid_batches(const P &p)
{
    if constexpr (HasBatch<P>::value) return p.batches(); else return 1;
}

// A problem type P provides:
//   using T                          operand type in LDS / MFMA (float or bf16_t)
//   static constexpr int BM, BN, BK  workgroup tile; WAVES_M in {1,2,4} wavefronts along M (4/WAVES_M along N)
//   static constexpr int VA, VB      elements fetched per load_a / load_b call
//   static constexpr bool A_ALONG_K, B_ALONG_K
//                                    true : the VA elements are k, k+1, ... of one row
//                                    false: the VA elements are rows row, row+1, ... at one k
//   int M, N, K, klen                logical sizes; blockIdx.y covers k in [y*klen, min(K,(y+1)*klen))
//   void load_a(int row, int k, int kend, float (&v)[VA]) const   zero-filled outside [0,M) x [.,kend)
//   void load_b(int col, int k, int kend, float (&v)[VB]) const
//   void store(int m, int n, float acc, int z) const              called only for m < M, n < N
template <class P>
__global__ __launch_bounds__(256) void gemm_kernel(const P p_in)
{
    P p = p_in;
    if constexpr (HasBatch<P>::value) p.set_batch(blockIdx.z);
    using T = typename P::T;
    using Tr = OperandTraits<T>;
    constexpr int BM = P::BM, BN = P::BN, BK = P::BK;
    constexpr int WM = P::WAVES_M, WN = 4 / WM;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int LS = BK + Tr::PAD;
    constexpr int VA = P::VA, VB = P::VB;
    constexpr int CA = BM * BK / VA, CB = BN * BK / VB;             // vectors per operand tile
    constexpr int NA = (CA + 255) / 256, NB = (CB + 255) / 256;     // vectors per thread (last one may be idle)
    static_assert(TM >= 1 && TN >= 1 && TM * 32 * WM == BM && TN * 32 * WN == BN, "tile shape");
    static_assert(CA * VA == BM * BK && CB * VB == BN * BK && BK % VA == 0 && BK % VB == 0 && BM % VA == 0 &&
                      BN % VB == 0, "loader shape");
    static_assert(BK % Tr::KINST == 0, "BK");
    constexpr int SEG = SegOf<P>::value;
    static_assert(SEG % BK == 0, "SEG must be a multiple of BK");

    __shared__ __attribute__((aligned(16))) T As[BM * LS];
    __shared__ __attribute__((aligned(16))) T Bs[BN * LS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int tiles_n = (p.N + BN - 1) / BN;
    const int m0 = (blockIdx.x / tiles_n) * BM, n0 = (blockIdx.x % tiles_n) * BN;
    if (m0 >= p.M) return;                 // a batch smaller than the largest one: the whole workgroup leaves
    const int z = blockIdx.y;
    const int kbeg = z * p.klen;
    const int kend = min(p.K, kbeg + p.klen);

    float ra[NA][VA], rb[NB][VB];

    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int id = tid + i * 256;
            if (CA % 256 != 0 && id >= CA) continue;
            if constexpr (P::A_ALONG_K) p.load_a(m0 + id / (BK / VA), k0 + (id % (BK / VA)) * VA, kend, ra[i]);
            else                        p.load_a(m0 + (id % (BM / VA)) * VA, k0 + id / (BM / VA), kend, ra[i]);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int id = tid + i * 256;
            if (CB % 256 != 0 && id >= CB) continue;
            if constexpr (P::B_ALONG_K) p.load_b(n0 + id / (BK / VB), k0 + (id % (BK / VB)) * VB, kend, rb[i]);
            else                        p.load_b(n0 + (id % (BN / VB)) * VB, k0 + id / (BN / VB), kend, rb[i]);
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int id = tid + i * 256;
            if (CA % 256 != 0 && id >= CA) continue;
            if constexpr (P::A_ALONG_K) {
                T *d = As + (id / (BK / VA)) * LS + (id % (BK / VA)) * VA;
#pragma unroll
                for (int j = 0; j < VA; ++j) d[j] = from_f32<T>(ra[i][j]);
            } else {
                T *d = As + ((id % (BM / VA)) * VA) * LS + id / (BM / VA);
#pragma unroll
                for (int j = 0; j < VA; ++j) d[j * LS] = from_f32<T>(ra[i][j]);
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int id = tid + i * 256;
            if (CB % 256 != 0 && id >= CB) continue;
            if constexpr (P::B_ALONG_K) {
                T *d = Bs + (id / (BK / VB)) * LS + (id % (BK / VB)) * VB;
#pragma unroll
                for (int j = 0; j < VB; ++j) d[j] = from_f32<T>(rb[i][j]);
            } else {
                T *d = Bs + ((id % (BN / VB)) * VB) * LS + id / (BN / VB);
#pragma unroll
                for (int j = 0; j < VB; ++j) d[j * LS] = from_f32<T>(rb[i][j]);
            }
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
    f32x16 tot[SEG > 0 ? TM : 1][SEG > 0 ? TN : 1];
    if constexpr (SEG > 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) tot[i][j][r] = 0.0f;
    }

    const int lrow = lane & 31, lk = lane >> 5;
    const T *a_base = As + (wm * TM * 32 + lrow) * LS;
    const T *b_base = Bs + (wn * TN * 32 + lrow) * LS;

    if (kbeg < kend) gload(kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        sstore();
        __syncthreads();
        if (k0 + BK < kend) gload(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK; kk += Tr::KINST) {
            if constexpr (sizeof(T) == 4) {
                float av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) av[i] = a_base[i * 32 * LS + kk + lk];
#pragma unroll
                for (int j = 0; j < TN; ++j) bv[j] = b_base[j * 32 * LS + kk + lk];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
            } else {
                bf16x8 av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    av[i] = *reinterpret_cast<const bf16x8 *>(a_base + i * 32 * LS + kk + lk * 8);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    bv[j] = *reinterpret_cast<const bf16x8 *>(b_base + j * 32 * LS + kk + lk * 8);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
        }
        if constexpr (SEG > 0) {
            if ((k0 + BK) % SEG == 0 || k0 + BK >= kend) {      // end of a segment: fold it into the running total
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) { tot[i][j][r] += acc[i][j][r]; acc[i][j][r] = 0.0f; }
            }
        }
        __syncthreads();
    }
    if constexpr (SEG > 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = tot[i][j];
    }

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + (wn * TN + j) * 32 + lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (m < p.M && n < p.N) p.store(m, n, acc[i][j][r], z);
            }
        }
}

template <class P> inline hipError_t launch_gemm(const P &p, hipStream_t stream)
{
    const int tiles = ((grid_rows(p) + P::BM - 1) / P::BM) * ((p.N + P::BN - 1) / P::BN);
    const int nz = (p.K + p.klen - 1) / p.klen;
    if (tiles <= 0 || nz <= 0) return hipSuccess;
    hipLaunchKernelGGL(gemm_kernel<P>, dim3(tiles, nz, grid_batches(p)), dim3(256, 1, 1), 0, stream, p);
    return hipGetLastError();
}

}  // namespace hts
