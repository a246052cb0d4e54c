// Tiled matrix-multiply core on CDNA4 matrix instructions (gfx950).
//
// Every dense contraction of the network (Nature-CNN of the paper's appendix "Implementation Details") is
// expressed as  D[m][n] = sum_k A(m,k) * B(n,k)  where a small "problem" object supplies the operand gathers
// (implicit im2col, index gather, weight layouts) and the epilogue (bias, ReLU, masks, output layout).
//
// One workgroup = WAVES_M x WAVES_N wavefronts of 64 lanes (2 to 8); each wavefront owns a (TM*32) x (TN*32) block of D
// built from 32x32 MFMA accumulators:
//   fp32 : v_mfma_f32_32x32x2_f32   (lane l supplies A[l%32][l/32] and B[l/32][l%32])
//   bf16 : v_mfma_f32_32x32x16_bf16 (lane l supplies 8 consecutive k at k0 = 8*(l/32) for row/col l%32)
// Accumulator register r of lane l is D[8*(r/4) + 4*(l/32) + r%4][l%32].
//
// Operand tiles go global -> registers -> LDS ([row][k], padded) -> MFMA; the global loads of tile i+1 are in
// flight while tile i is multiplied.  Gathers are separable: the part of an address that depends on the tile row
// (batch / y / x decomposition, done with multiply-shift division) is computed once per thread before the K loop
// (ctx_a / ctx_b); the part that depends on k is cheap.  blockIdx.y selects a contiguous K range of length p.klen
// (split-K); the problem's store() receives that index so partial sums go to distinct slots and are later combined
// in a fixed order (no atomics anywhere).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>
#include <utility>

#define HTS_HD __host__ __device__ __forceinline__

namespace hts {

typedef __bf16 bf16_t;
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T, int V> struct VecOf { typedef T type __attribute__((ext_vector_type(V))); };
template <typename T> struct VecOf<T, 1> {
    struct type {
        T x;
        HTS_HD T &operator[](int) { return x; }
        HTS_HD const T &operator[](int) const { return x; }
    };
};
template <typename T, int V> using Vec = typename VecOf<T, V>::type;
typedef Vec<bf16_t, 8> bf16x8;

template <typename T> struct OperandTraits;
template <> struct OperandTraits<float> {
    static constexpr int KINST = 2;   // k consumed per MFMA
    static constexpr int PAD = 1;     // LDS row padding (elements); rows are written element by element
    static constexpr int VEC = 4;     // elements per 16-byte global access
    static constexpr int BK = 32;     // k per staged tile
};
template <> struct OperandTraits<bf16_t> {
    static constexpr int KINST = 16;
    static constexpr int PAD = 8;     // keeps rows 16-byte aligned and spreads them over the banks
    static constexpr int VEC = 8;
    static constexpr int BK = 64;
};

HTS_HD float to_f32(float x) { return x; }
HTS_HD float to_f32(bf16_t x) { return (float)x; }
template <typename T> HTS_HD T from_f32(float x);
template <> HTS_HD float from_f32<float>(float x) { return x; }
template <> HTS_HD bf16_t from_f32<bf16_t>(float x) { return (bf16_t)x; }   // round to nearest even

// Exact floor(x / d) for 0 <= x < 2^31 by multiply-shift: mul = ceil(2^p / d), p = 31 + ceil(log2 d).
struct FastDiv {
    uint32_t mul;
    int shr, d;
    static inline FastDiv make(int d)
    {
        FastDiv f;
        f.d = d < 1 ? 1 : d;
        int lg = 0;
        while ((1ll << lg) < f.d) ++lg;
        const int p = 31 + lg;
        f.mul = (uint32_t)(((1ull << p) + (unsigned long long)f.d - 1) / (unsigned long long)f.d);
        f.shr = p - 32 < 0 ? 0 : p - 32;        // d == 1 (p = 31) is answered by the select below
        return f;
    }
    HTS_HD int div(int x) const                 // a select, not a branch: a branch would end the basic block and with it
    {                                           // the window in which loads around the division can be issued together
#if defined(__HIP_DEVICE_COMPILE__)
        const int q = (int)(__umulhi((uint32_t)x, mul) >> shr);
#else
        const int q = (int)((((unsigned long long)(uint32_t)x * mul) >> 32) >> shr);
#endif
        return d == 1 ? x : q;
    }
};

// contiguous loads of V operands of type T from memory of type S (conversion to T happens here)
template <typename T, int V> HTS_HD Vec<T, V> zero_vec()
{
    Vec<T, V> v;
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] = from_f32<T>(0.0f);
    return v;
}
template <typename T, int V, typename S> HTS_HD Vec<T, V> load_vec(const S *p)
{
    if constexpr (std::is_same<S, T>::value) return *reinterpret_cast<const Vec<T, V> *>(p);
    else {
        const Vec<S, V> s = *reinterpret_cast<const Vec<S, V> *>(p);
        Vec<T, V> v;
#pragma unroll
        for (int i = 0; i < V; ++i) v[i] = from_f32<T>(to_f32(s[i]));
        return v;
    }
}
// v where keep, zeros otherwise, as selects on whole registers.  Loaders fetch from a clamped (always valid) address
// and mask afterwards: a load inside a branch would have to be waited for before the next branch is entered, which
// puts one memory round trip after the other.
template <typename T, int V> HTS_HD Vec<T, V> keep_if(bool keep, const Vec<T, V> &v)
{
    if constexpr (V == 1) { Vec<T, V> r; r[0] = keep ? v[0] : from_f32<T>(0.0f); return r; }
    else {
        constexpr int N = V * (int)sizeof(T) / 4;
        static_assert(N >= 1 && N * 4 == V * (int)sizeof(T), "whole registers");
        if constexpr (N == 1) {
            const uint32_t w = __builtin_bit_cast(uint32_t, v);
            return __builtin_bit_cast(Vec<T, V>, keep ? w : 0u);
        } else {
            typedef uint32_t words __attribute__((ext_vector_type(N)));
            words w = __builtin_bit_cast(words, v);
#pragma unroll
            for (int i = 0; i < N; ++i) w[i] = keep ? w[i] : 0u;
            return __builtin_bit_cast(Vec<T, V>, w);
        }
    }
}
// 8 bytes (4-byte aligned) as 8 operands
template <typename T> HTS_HD Vec<T, 8> load_u8x8(const uint8_t *p)
{
    const uint32_t lo = *reinterpret_cast<const uint32_t *>(p), hi = *reinterpret_cast<const uint32_t *>(p + 4);
    Vec<T, 8> v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[i] = from_f32<T>((float)((lo >> (8 * i)) & 0xFFu));
        v[4 + i] = from_f32<T>((float)((hi >> (8 * i)) & 0xFFu));
    }
    return v;
}

// Optional segmented accumulation: a problem that defines `static constexpr int SEG` (a multiple of BK) gets
//   D = (((s_0 + s_1) + s_2) + ...),  s_i = MFMA-accumulated sum over k in [i*SEG, (i+1)*SEG)
// instead of one long accumulation chain.  The wave-per-segment kernel of wsgemm.hpp computes the s_i in parallel
// and adds them in the same order, so both kernels return identical bits for the same problem.
template <class P, class = void> struct SegOf { static constexpr int value = 0; };
template <class P> struct SegOf<P, std::void_t<decltype(P::SEG)>> { static constexpr int value = P::SEG; };

// Optional second level: a problem that also defines `static constexpr int GROUP` (a multiple of SEG) has the segment
// sums of each group of GROUP reduction indices added up first and the group sums then added in group order,
//   D = (((0 + g_0) + g_1) + ...),  g_j = ((s_0 + s_1) + ...) over the segments of group j
// -- what a consumer computes that receives one partial per group (klen = GROUP) and adds them in order, so a launch
// may cover any whole number of groups per reduction chunk without changing a bit of the result.
template <class P, class = void> struct GroupOf { static constexpr int value = 0; };
template <class P> struct GroupOf<P, std::void_t<decltype(P::GROUP)>> { static constexpr int value = P::GROUP; };

// Optional prefetch depth: a problem that defines `static constexpr int STAGES = D` keeps the global loads of D k-tiles
// in flight in registers (default 1: the next tile only).  The order of the arithmetic does not change.
template <class P, class = void> struct StagesOf { static constexpr int value = 1; };
template <class P> struct StagesOf<P, std::void_t<decltype(P::STAGES)>> { static constexpr int value = P::STAGES; };

// Optional: a problem with `static constexpr bool STEADY = true` (and no SEG) gets a k loop whose whole groups of
// steps load unconditionally, with the end-of-range checks folded away; the last steps keep the checks.
template <class P, class = void> struct SteadyOf { static constexpr bool value = false; };
template <class P> struct SteadyOf<P, std::void_t<decltype(P::STEADY)>> { static constexpr bool value = P::STEADY; };

// Optional "lane owns a row" orientation: a problem with `static constexpr bool LANE_OWNS_ROW = true` has the two
// operands of the matrix instruction exchanged, so that a lane's 16 accumulator registers are 16 columns (four groups
// of four neighbours) of ONE output row instead of 16 rows of one column.  Its epilogue then needs one row context
// per lane (`Row row(int m[, int batch]) const`: e.g. a position decomposition) and stores four neighbouring columns
// at a time: `Pre pre4(const Row &, int n) const` fetches what the store needs from memory (bias, mask) and
// `store4(const Row &, int n, const float (&v)[4], int z[, int batch], const Pre &) const` finishes; n and N are
// multiples of 4.
template <class P, class = void> struct OwnsRow : std::false_type {};
template <class P> struct OwnsRow<P, std::void_t<decltype(P::LANE_OWNS_ROW)>> : std::integral_constant<bool, P::LANE_OWNS_ROW> {};

// Optional natural staging of operands that are contiguous along the row index instead of along the reduction (the
// weight gradients): a problem with `static constexpr bool NATURAL_LDS = true` has such an operand loaded by threads
// whose neighbours take neighbouring row vectors at ONE reduction index (whole cache lines per load instruction), kept in
// LDS as it lies in memory ([reduction][row], padded), and brought into the matrix instruction's lane layout by the
// transposing LDS read (bf16) or by plain element reads (fp32).  No register transposes; same operand values in the
// same lanes as the default staging, hence the same bits.
template <class P, class = void> struct NaturalOf : std::false_type {};
template <class P> struct NaturalOf<P, std::void_t<decltype(P::NATURAL_LDS)>> : std::integral_constant<bool, P::NATURAL_LDS> {};
typedef short i16x4 __attribute__((ext_vector_type(4)));

// Optional run loaders for operands that are contiguous along the reduction instead of along k: a problem with
// `void load_a_run(const CtxA &, int k, int kend, Vec<T,VA> (&out)[VA]) const` (likewise load_b_run) fetches the VA
// vectors of k, k+1, ..., k+VA-1 in one call, so the decomposition of k is done once and advanced incrementally.
template <class P, class = void> struct HasRunA : std::false_type {};
template <class P> struct HasRunA<P, std::void_t<decltype(&P::load_a_run)>> : std::true_type {};
template <class P, class = void> struct HasRunB : std::false_type {};
template <class P> struct HasRunB<P, std::void_t<decltype(&P::load_b_run)>> : std::true_type {};

// Optional batching: a problem with `int batches() const`, `int max_m() const`, `int batch_m(int z) const` is
// launched with gridDim.z = batches(); batch z has batch_m(z) rows and its own gathers: ctx_a(row, z),
// ctx_b(col, z) and store(m, n, acc, split, z) receive the batch index (the problem object stays read-only).
// Optional tile order (see the kernel): N slowest instead of M slowest.
template <class P, class = void> struct TilesAlongM : std::false_type {};
template <class P> struct TilesAlongM<P, std::void_t<decltype(P::TILES_ALONG_M)>> : std::integral_constant<bool, P::TILES_ALONG_M> {};

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
template <class P> HTS_HD int rows_of(const P &p, int zb)
{
    if constexpr (HasBatch<P>::value) return p.batch_m(zb); else return p.M;
}
template <class P> HTS_HD typename P::CtxA make_ctx_a(const P &p, int row, int zb)
{
    if constexpr (HasBatch<P>::value) return p.ctx_a(row, zb); else return p.ctx_a(row);
}
template <class P> HTS_HD typename P::CtxB make_ctx_b(const P &p, int col, int zb)
{
    if constexpr (HasBatch<P>::value) return p.ctx_b(col, zb); else return p.ctx_b(col);
}
// Optional per-column epilogue data: a problem with `Col col(int n) const` (n < N) has it evaluated once per
// output column held by a lane (e.g. the bias) and receives it as the last argument of store().
template <class P, class = void> struct HasCol : std::false_type {};
template <class P> struct HasCol<P, std::void_t<decltype(std::declval<const P &>().col(0))>> : std::true_type {};
struct NoCol {};
template <class P> HTS_HD auto make_col(const P &p, int n)
{
    if constexpr (HasCol<P>::value) return p.col(n); else return NoCol{};
}
template <class P, class C> HTS_HD void do_store(const P &p, int m, int n, float acc, int z, int zb, const C &col)
{
    if constexpr (HasCol<P>::value) {
        if constexpr (HasBatch<P>::value) p.store(m, n, acc, z, zb, col); else p.store(m, n, acc, z, col);
    } else {
        if constexpr (HasBatch<P>::value) p.store(m, n, acc, z, zb); else p.store(m, n, acc, z);
    }
}

// Optional element-wise form of the same idea for the wave-per-segment kernel: `Pre1 pre1(int m, int n[, int batch])`
// fetches what one output element's store needs (its address, a ReLU mask) and `store1(const Pre1 &, float acc)`
// finishes; pre1() is called at kernel start, store1() when the sums are ready.
template <class P, class = void> struct HasPre1 : std::false_type {};
template <class P> struct HasPre1<P, std::void_t<decltype(&P::store1)>> : std::true_type {};
template <class P, bool> struct Pre1Type { typedef int type; };
template <class P> struct Pre1Type<P, true> { typedef typename P::Pre1 type; };
template <class P> HTS_HD auto epi_pre1(const P &p, int m, int n, int zb)
{
    if constexpr (HasBatch<P>::value) return p.pre1(m, n, zb); else return p.pre1(m, n);
}

// Epilogue inputs of a "lane owns a row" problem (row contexts, and what pre4() fetches: bias, ReLU masks).  They
// are requested BEFORE the k loop and held in registers, so that they travel while the products are formed; fetched
// after the loop, every workgroup would end with a bare memory round trip.
template <class P> HTS_HD auto epi_row(const P &p, int mr, int zb)
{
    if constexpr (HasBatch<P>::value) return p.row(mr, zb); else return p.row(mr);
}
// (A problem whose pre4() only reads a few hot bytes -- a bias -- opts out with `static constexpr bool
// EPI_INPUTS_EARLY = false`: its registers are better left to the k loop, and the fetch then precedes the stores.)
template <class P, class = void> struct EpiEarly : std::true_type {};
template <class P> struct EpiEarly<P, std::void_t<decltype(P::EPI_INPUTS_EARLY)>> : std::integral_constant<bool, P::EPI_INPUTS_EARLY> {};
template <class P, int TM, int TN, bool SWAP> struct EpiInputs {};
template <class P, int TM, int TN> struct EpiInputs<P, TM, TN, true> {
    using RowT = decltype(epi_row(std::declval<const P &>(), 0, 0));
    using PreT = decltype(std::declval<const P &>().pre4(std::declval<const RowT &>(), 0));
    RowT rc[TM];
    PreT pre[TM][TN][4];
    bool mok[TM];
};

// A problem type P provides:
//   using T                          operand type in LDS / MFMA (float or bf16_t)
//   static constexpr int BM, BN, BK  workgroup tile; WAVES_M x WAVES_N wavefronts (64 lanes each) share it
//   static constexpr int VA, VB      operands fetched per load_a / load_b call
//   static constexpr bool A_ALONG_K, B_ALONG_K
//                                    true : the VA operands are k, k+1, ... of one row
//                                    false: the VA operands are rows row, row+1, ... at one k; a thread then fetches
//                                           VA consecutive k and transposes the VA x VA block in registers, so
//                                           that LDS rows are still written as whole k-contiguous vectors
//   int M, N, K, klen                logical sizes; blockIdx.y covers k in [y*klen, min(K,(y+1)*klen))
//   CtxA ctx_a(int row) const        row-dependent part of the gather (row = first row of the vector)
//   Vec<T,VA> load_a(const CtxA &, int k, int kend) const     zero outside [0,M) x [.,kend)
//   CtxB ctx_b(int col) const,  Vec<T,VB> load_b(const CtxB &, int k, int kend) const
//   void store(int m, int n, float acc, int z) const          called only for m < M, n < N
//   optionally Col col(int n) const and store(..., const Col &)   per-column epilogue data, fetched once per lane
template <class P>
__global__ __launch_bounds__(P::WAVES_M * P::WAVES_N * 64) void gemm_kernel(const P p)
{
    const int zb = blockIdx.z, M = rows_of(p, zb);
    using T = typename P::T;
    using Tr = OperandTraits<T>;
    constexpr int BM = P::BM, BN = P::BN, BK = P::BK;
    constexpr int WM = P::WAVES_M, WN = P::WAVES_N, NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int LS = BK + Tr::PAD;
    constexpr int VA = P::VA, VB = P::VB;
    // natural staging ([reduction][row + pad]); the pad keeps the row pitch at 64 bytes modulo 128 for bf16 (the four
    // reduction rows a 16-lane group reads at once fall into different banks) and 128 modulo 256 for fp32
    constexpr bool NAT_A = NaturalOf<P>::value && !P::A_ALONG_K, NAT_B = NaturalOf<P>::value && !P::B_ALONG_K;
    constexpr int LSNA = BM + (BM % 64 == 0 ? 32 : 0), LSNB = BN + (BN % 64 == 0 ? 32 : 0);
    // work items per operand tile: a k-contiguous vector (ALONG_K), a row-contiguous vector at one reduction index
    // (natural staging) or a V x V block to transpose (otherwise)
    constexpr int CA = P::A_ALONG_K ? BM * BK / VA : (NAT_A ? BK * (BM / VA) : (BM / VA) * (BK / VA));
    constexpr int CB = P::B_ALONG_K ? BN * BK / VB : (NAT_B ? BK * (BN / VB) : (BN / VB) * (BK / VB));
    constexpr int NA = (CA + NT - 1) / NT, NB = (CB + NT - 1) / NT;     // items per thread (last one may be idle)
    constexpr int RA = (P::A_ALONG_K || NAT_A) ? 1 : VA, RB = (P::B_ALONG_K || NAT_B) ? 1 : VB; // vectors held per item
    static_assert(TM >= 1 && TN >= 1 && TM * 32 * WM == BM && TN * 32 * WN == BN, "tile shape");
    static_assert(BK % VA == 0 && BK % VB == 0 && BM % VA == 0 && BN % VB == 0, "loader shape");
    static_assert(BK % Tr::KINST == 0, "BK");
    constexpr int SEG = SegOf<P>::value;
    static_assert(SEG % BK == 0, "SEG must be a multiple of BK");
    constexpr bool VEC_LDS = sizeof(T) == 2;      // bf16 rows are 16-byte aligned: whole vectors are stored at once

    __shared__ __attribute__((aligned(16))) T As[NAT_A ? BK * LSNA : BM * LS];
    __shared__ __attribute__((aligned(16))) T Bs[NAT_B ? BK * LSNB : BN * LS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int tiles_n = (p.N + BN - 1) / BN;
    int tile = blockIdx.x, z = blockIdx.y;
    if constexpr (!HasBatch<P>::value) {
        // A long split reduction is launched as a one-dimensional grid (see launch_gemm): workgroups go to the eight
        // XCDs in turn, so workgroup h runs on XCD h % 8; all output tiles of reduction chunk z are given to XCD z % 8,
        // whose L2 then serves the operand rows that those tiles share.
        if (gridDim.y == 1 && p.klen < p.K) {
            const int tiles = ((M + BM - 1) / BM) * tiles_n;
            const int xcd = tile & 7, slot = tile >> 3;
            z = (slot / tiles) * 8 + xcd;
            tile = slot % tiles;
            if ((long long)z * p.klen >= p.K) return;        // padding of the last round of eight chunks
        } else {
            // Otherwise gridDim.x is the number of tiles rounded up to a multiple of 8, and XCD x takes the x-th
            // eighth of the tile order: neighbouring tiles share an operand panel, and a panel that is needed on one
            // XCD only is fetched into one L2 only.  (Round-robin, every XCD read the whole of the operand that the
            // tile order walks slowest: the FC forward pass fetched its activations eight times, 107 MB for 34.)
            // (A single column of tiles shares nothing but the small weight panel and keeps the round-robin order.)
            const int tiles = ((M + BM - 1) / BM) * tiles_n, per_xcd = gridDim.x >> 3;
            if (tiles_n > 1) tile = (tile & 7) * per_xcd + (tile >> 3);
            if (tile >= tiles) return;
        }
    }
    // the tile order walks N fastest, so an XCD's share is a range of rows and all columns; a problem whose column
    // operand is the larger one asks for the transposed order (`static constexpr bool TILES_ALONG_M = true`)
    int m0, n0;
    if constexpr (TilesAlongM<P>::value) {
        const int tiles_m = (M + BM - 1) / BM;
        m0 = (tile % tiles_m) * BM; n0 = (tile / tiles_m) * BN;
    } else {
        m0 = (tile / tiles_n) * BM; n0 = (tile % tiles_n) * BN;
    }
    if (m0 >= M) return;                   // a batch smaller than the largest one: the whole workgroup leaves
    const int kbeg = z * p.klen;
    const int kend = min(p.K, kbeg + p.klen);

    // fixed assignment of operand items to threads; the row part of every gather is resolved once
    typename P::CtxA ca[NA];
    typename P::CtxB cb[NB];
    int ka[NA], kb[NB], la[NA], lb[NB];          // k offset inside the tile, LDS offset
#pragma unroll
    // When an operand tile has fewer items than the workgroup has threads (or a last, partial round of them), the
    // spare threads repeat other threads' items -- same loads, same LDS stores of the same values -- instead of
    // sitting out: an `if (owns an item)` around a store puts the store in a branch, and in a branch the compiler
    // waits for EVERY outstanding load, the prefetched tile's included (conv1 on 16-channel frames, whose weight tile
    // has 256 items for 512 threads, stalled 1600 cycles every second k-tile that way).
    for (int i = 0; i < NA; ++i) {
        const int id = CA % NT == 0 ? tid + i * NT : (tid + i * NT) % CA;
        int r;
        if constexpr (P::A_ALONG_K) { r = id / (BK / VA); ka[i] = (id % (BK / VA)) * VA; }
        else if constexpr (NAT_A) { r = (id % (BM / VA)) * VA; ka[i] = id / (BM / VA); }
        else { r = (id / (BK / VA)) * VA; ka[i] = (id % (BK / VA)) * VA; }     // neighbours write one LDS row
        la[i] = NAT_A ? ka[i] * LSNA + r : r * LS + ka[i];
        ca[i] = make_ctx_a(p, m0 + r, zb);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int id = CB % NT == 0 ? tid + i * NT : (tid + i * NT) % CB;
        int r;
        if constexpr (P::B_ALONG_K) { r = id / (BK / VB); kb[i] = (id % (BK / VB)) * VB; }
        else if constexpr (NAT_B) { r = (id % (BN / VB)) * VB; kb[i] = id / (BN / VB); }
        else { r = (id / (BK / VB)) * VB; kb[i] = (id % (BK / VB)) * VB; }
        lb[i] = NAT_B ? kb[i] * LSNB + r : r * LS + kb[i];
        cb[i] = make_ctx_b(p, n0 + r, zb);
    }

    constexpr int D = StagesOf<P>::value;
    constexpr bool SWAP = OwnsRow<P>::value;
    static_assert(D >= 1 && D <= 4, "prefetch depth");
    Vec<T, VA> rra[D][NA][RA];
    Vec<T, VB> rrb[D][NB][RB];
    // lim = end of the reduction range for this load, or INT_MAX when the whole k-tile is known to lie inside it
    // (the range checks then fold away and the loads are unconditional)
    auto gload = [&](int k0, Vec<T, VA> (&ra)[NA][RA], Vec<T, VB> (&rb)[NB][RB], int lim) {
#pragma unroll
        for (int i = 0; i < NA; ++i)
            {
                if constexpr (!P::A_ALONG_K && !NAT_A && HasRunA<P>::value) p.load_a_run(ca[i], k0 + ka[i], lim, ra[i]);
                else {
#pragma unroll
                    for (int q = 0; q < RA; ++q) ra[i][q] = p.load_a(ca[i], k0 + ka[i] + q, lim);
                }
            }
#pragma unroll
        for (int i = 0; i < NB; ++i)
            {
                if constexpr (!P::B_ALONG_K && !NAT_B && HasRunB<P>::value) p.load_b_run(cb[i], k0 + kb[i], lim, rb[i]);
                else {
#pragma unroll
                    for (int q = 0; q < RB; ++q) rb[i][q] = p.load_b(cb[i], k0 + kb[i] + q, lim);
                }
            }
    };
    auto sstore = [&](const Vec<T, VA> (&ra)[NA][RA], const Vec<T, VB> (&rb)[NB][RB]) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            T *d = As + la[i];
            if constexpr (NAT_A) *reinterpret_cast<Vec<T, VA> *>(d) = ra[i][0];
            else if constexpr (P::A_ALONG_K) {
                if constexpr (VEC_LDS) *reinterpret_cast<Vec<T, VA> *>(d) = ra[i][0];
                else {
#pragma unroll
                    for (int j = 0; j < VA; ++j) d[j] = ra[i][0][j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < VA; ++j) {          // row r+j gets the k-contiguous vector (block column j)
                    Vec<T, VA> t;
#pragma unroll
                    for (int q = 0; q < VA; ++q) t[q] = ra[i][q][j];
                    if constexpr (VEC_LDS) *reinterpret_cast<Vec<T, VA> *>(d + j * LS) = t;
                    else {
#pragma unroll
                        for (int q = 0; q < VA; ++q) d[j * LS + q] = t[q];
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            T *d = Bs + lb[i];
            if constexpr (NAT_B) *reinterpret_cast<Vec<T, VB> *>(d) = rb[i][0];
            else if constexpr (P::B_ALONG_K) {
                if constexpr (VEC_LDS) *reinterpret_cast<Vec<T, VB> *>(d) = rb[i][0];
                else {
#pragma unroll
                    for (int j = 0; j < VB; ++j) d[j] = rb[i][0][j];
                }
            } else {
#pragma unroll
                for (int j = 0; j < VB; ++j) {
                    Vec<T, VB> t;
#pragma unroll
                    for (int q = 0; q < VB; ++q) t[q] = rb[i][q][j];
                    if constexpr (VEC_LDS) *reinterpret_cast<Vec<T, VB> *>(d + j * LS) = t;
                    else {
#pragma unroll
                        for (int q = 0; q < VB; ++q) d[j * LS + q] = t[q];
                    }
                }
            }
        }
    };

    const int lrow = lane & 31, lk = lane >> 5;
    const T *a_base = As + (wm * TM * 32 + lrow) * LS;
    const T *b_base = Bs + (wn * TN * 32 + lrow) * LS;
    // Natural staging, bf16: the transposing read works on groups of 16 lanes; lane 4j+q of a group points at 4 row
    // entries (4q..4q+3 of the group's 16) of reduction index j (< 4) and receives the 4 reduction indices of row
    // entry (lane % 16).  Groups 0,1 cover rows 0-15 and 16-31 at reduction 0-7 (two reads), groups 2,3 at 8-15.
    // fp32: lane (row, k) reads its element.
    const int nat_off_a = sizeof(T) == 2 ? (8 * (lane >> 5) + ((lane & 15) >> 2)) * LSNA + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)
                                         : lk * LSNA + lrow;
    const int nat_off_b = sizeof(T) == 2 ? (8 * (lane >> 5) + ((lane & 15) >> 2)) * LSNB + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)
                                         : lk * LSNB + lrow;
    const T *a_nat = As + wm * TM * 32 + nat_off_a;
    const T *b_nat = Bs + wn * TN * 32 + nat_off_b;
    auto tr8 = [](const T *q, int pitch) {      // 8 reduction indices of one row entry: two transposing reads
        typedef i16x4 __attribute__((address_space(3))) *lds_ptr;
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q));
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(q + 4 * pitch));
        typedef short i16x8 __attribute__((ext_vector_type(8)));
        const i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, v);
    };

    // one k-tile: registers -> LDS, refill this stage's registers with the tile D steps ahead, multiply.
    // REFILL: 1 = always (steady state: an unconditional load lets the compiler wait for exactly the older stages),
    // 0 = never, 2 = if that tile exists
    auto step_s = [&](int k0, f32x16 (&acc)[TM][TN], Vec<T, VA> (&ra)[NA][RA], Vec<T, VB> (&rb)[NB][RB], auto refill) {
        constexpr int REFILL = decltype(refill)::value;
        sstore(ra, rb);
        __syncthreads();
        if constexpr (REFILL == 1) gload(k0 + D * BK, ra, rb, 0x7fffffff);
        else if constexpr (REFILL == 2) { if (k0 + D * BK < kend) gload(k0 + D * BK, ra, rb, kend); }
#pragma unroll
        for (int kk = 0; kk < BK; kk += Tr::KINST) {
            if constexpr (sizeof(T) == 4) {
                float av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) av[i] = NAT_A ? a_nat[kk * LSNA + i * 32] : a_base[i * 32 * LS + kk + lk];
#pragma unroll
                for (int j = 0; j < TN; ++j) bv[j] = NAT_B ? b_nat[kk * LSNB + j * 32] : b_base[j * 32 * LS + kk + lk];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x2f32(bv[j], av[i], acc[i][j], 0, 0, 0)
                                         : __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
            } else {
                bf16x8 av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if constexpr (NAT_A) av[i] = tr8(a_nat + kk * LSNA + i * 32, LSNA);
                    else av[i] = *reinterpret_cast<const bf16x8 *>(a_base + i * 32 * LS + kk + lk * 8);
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (NAT_B) bv[j] = tr8(b_nat + kk * LSNB + j * 32, LSNB);
                    else bv[j] = *reinterpret_cast<const bf16x8 *>(b_base + j * 32 * LS + kk + lk * 8);
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv[j], av[i], acc[i][j], 0, 0, 0)
                                         : __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
        }
        __syncthreads();
    };
    auto clear = [&](f32x16 (&x)[TM][TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) x[i][j][r] = 0.0f;
    };

    f32x16 acc[TM][TN];
    clear(acc);
    // (unconditional: a stage beyond the end of a short reduction range fetches the range's last k-tile once more and
    // is never consumed -- a branch here leaves the compiler unsure how many loads are outstanding when the k loop
    // starts, and it then waits for all of them at the top of every iteration)
#pragma unroll
    for (int s = 0; s < D; ++s) {
        const int last = kbeg + ((kend - kbeg - 1) / BK) * BK;
        gload(min(kbeg + s * BK, last), rra[s], rrb[s], kend);
    }
    EpiInputs<P, TM, TN, SWAP> epi;
    auto fetch_epi = [&]() {
        if constexpr (SWAP) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int m = m0 + (wm * TM + i) * 32 + lrow;
                epi.mok[i] = m < M;
                epi.rc[i] = epi_row(p, epi.mok[i] ? m : M - 1, zb);
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        epi.pre[i][j][g] = p.pre4(epi.rc[i], min(n0 + (wn * TN + j) * 32 + 8 * g + 4 * lk, p.N - 4));
            }
        }
    };
    if constexpr (SWAP && EpiEarly<P>::value) fetch_epi();
    if constexpr (D > 1 || (SEG == 0 && SteadyOf<P>::value)) {
        // the k loop is unrolled by the depth so that every stage has its own registers; whole groups of steps
        // refill unconditionally
        f32x16 sacc[TM][TN];
        clear(sacc);
        auto fold = [&](int k0) {
            if (SEG == 0 ? k0 + BK >= kend : ((k0 + BK - kbeg) % (SEG > 0 ? SEG : 1) == 0 || k0 + BK >= kend)) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) { acc[i][j][r] += sacc[i][j][r]; sacc[i][j][r] = 0.0f; }
            }
        };
        int kg = kbeg;
        // steady state: whole groups of D steps, each of which refills its stage
        for (; kg + 2 * D * BK <= kend; kg += D * BK) {
#pragma unroll
            for (int s = 0; s < D; ++s) {
                step_s(kg + s * BK, sacc, rra[s], rrb[s], std::integral_constant<int, 1>{});
                fold(kg + s * BK);
            }
        }
        // the last (at most 2 D) steps
        for (; kg < kend; kg += D * BK) {
#pragma unroll
            for (int s = 0; s < D; ++s) {
                const int k0 = kg + s * BK;
                if (k0 >= kend) break;                 // uniform over the workgroup
                step_s(k0, sacc, rra[s], rrb[s], std::integral_constant<int, 2>{});
                fold(k0);
            }
        }
    } else if constexpr (SEG > 0) {
        auto step = [&](int k0, f32x16 (&a)[TM][TN]) { step_s(k0, a, rra[0], rrb[0], std::integral_constant<int, 2>{}); };
        // one fresh accumulator per segment (it only lives inside the segment), folded into the running total
        constexpr int SPS = SEG / BK;            // k-tiles per segment
        constexpr int GROUP = GroupOf<P>::value;
        static_assert(GROUP % SEG == 0, "a group is a whole number of segments");
        f32x16 tot[GROUP > 0 ? TM : 1][GROUP > 0 ? TN : 1];      // running sum of the finished groups
        if constexpr (GROUP > 0) clear(tot);
        auto close_group = [&]() {
            if constexpr (GROUP > 0) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int r = 0; r < 16; ++r) { tot[i][j][r] += acc[i][j][r]; acc[i][j][r] = 0.0f; }
            }
        };
        int k0 = kbeg;
        for (; k0 + SEG <= kend; k0 += SEG) {
            f32x16 sacc[TM][TN];
            clear(sacc);
#pragma unroll
            for (int s = 0; s < SPS; ++s) step(k0 + s * BK, sacc);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += sacc[i][j][r];
            if constexpr (GROUP > 0) {
                if ((k0 + SEG - kbeg) % GROUP == 0) close_group();
            }
        }
        if (k0 < kend) {                          // a last, shorter segment
            f32x16 sacc[TM][TN];
            clear(sacc);
            for (; k0 < kend; k0 += BK) step(k0, sacc);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += sacc[i][j][r];
        }
        if constexpr (GROUP > 0) {
            if ((kend - kbeg) % GROUP != 0) close_group();      // a last, shorter group
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = tot[i][j];
        }
    } else {
        for (int k0 = kbeg; k0 < kend; k0 += BK) step_s(k0, acc, rra[0], rrb[0], std::integral_constant<int, 2>{});
    }

    // Epilogue.  Tiles that lie wholly inside the output take a branch-free path (the compiler can then batch the
    // loads an epilogue may need); edge tiles check every element.
    auto epilogue = [&](auto full_tile) {
        constexpr bool FULL = decltype(full_tile)::value;
        if constexpr (SWAP) {
            if constexpr (!EpiEarly<P>::value) fetch_epi();
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int n = n0 + (wn * TN + j) * 32 + 8 * g + 4 * lk;
                        const float v[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                        if (FULL || (epi.mok[i] && n < p.N)) {
                            if constexpr (HasBatch<P>::value) p.store4(epi.rc[i], n, v, z, zb, epi.pre[i][j][g]);
                            else p.store4(epi.rc[i], n, v, z, epi.pre[i][j][g]);
                        }
                    }
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = n0 + (wn * TN + j) * 32 + lrow;
                    const auto col = make_col(p, FULL ? n : min(n, p.N - 1));
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * lk + (r % 4);
                        if (FULL || (m < M && n < p.N)) do_store(p, m, n, acc[i][j][r], z, zb, col);
                    }
                }
        }
    };
    if (m0 + BM <= M && n0 + BN <= p.N) epilogue(std::true_type{}); else epilogue(std::false_type{});
}

template <class P> inline hipError_t launch_gemm(const P &p, hipStream_t stream)
{
    const int tiles = ((grid_rows(p) + P::BM - 1) / P::BM) * ((p.N + P::BN - 1) / P::BN);
    const int nz = (p.K + p.klen - 1) / p.klen;
    if (tiles <= 0 || nz <= 0) return hipSuccess;
    dim3 grid(tiles, nz, grid_batches(p));
    if constexpr (!HasBatch<P>::value) {
        if (nz >= 32) grid = dim3(((nz + 7) / 8) * 8 * tiles, 1, 1);      // XCD-aware order, decoded in the kernel
        else grid.x = ((tiles + 7) / 8) * 8;                              // likewise: an eighth of the tiles per XCD
    }
    hipLaunchKernelGGL(gemm_kernel<P>, grid, dim3(P::WAVES_M * P::WAVES_N * 64, 1, 1), 0, stream, p);
    return hipGetLastError();
}

}  // namespace hts
