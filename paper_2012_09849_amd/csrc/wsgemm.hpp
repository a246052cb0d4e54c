// Wave-per-segment contraction for small problems (few rows, as in an actor's batch of 16-32 observations).
//
// The tile kernel of gemm.hpp walks K in one dependent chain per workgroup; with a handful of workgroups that chain
// (global-load latency + 64-cycle fp32 MFMAs) is the whole run time.  Here every wavefront owns one 32x32 output
// tile and ONE K segment of SEG elements: it fetches its two 32xSEG operand panels in a single burst, multiplies
// them, and the segment sums of a tile are added in segment order,
//     D = (((s_0 + s_1) + s_2) + ...),
// exactly the order the tile kernel uses for a problem with the same SEG -- results are bit-identical.
//
// Two forms:
//   PARTIAL = false  workgroup (tile, y) owns the segments [y*spg, (y+1)*spg) of its tile (spg = segments per group,
//                    a launch argument; spg >= number of segments means one group).  Its WAVES wavefronts take them
//                    in rounds of WAVES; after each round the partial tiles go through LDS and are folded into the
//                    running total in wave order; the epilogue p.store(m, n, total, y) runs once.
//   PARTIAL = true   every wavefront stores its segment sum with p.store(m, n, s_seg, seg); the consumer adds the
//                    partials in segment order (used when K is too long for one workgroup, i.e. the FC layer).
#pragma once
#include "gemm.hpp"

namespace hts {

// BDIR = true (needs B_ALONG_K): the B operand (a weight matrix, rows contiguous in k) skips LDS -- every lane
// loads the k-vectors of its own column straight into registers and picks the elements its MFMA slot needs.  That
// halves the LDS footprint, so twice as many wavefronts (segments) fit in one workgroup.
template <class P, int WAVES, int SEG, bool PARTIAL, bool BDIR = false>
__global__ __launch_bounds__(WAVES * 64) void wsgemm_kernel(const P p, const int spg)
{
    static_assert(!BDIR || P::B_ALONG_K, "direct B operands must be contiguous along k");
    const int zb = blockIdx.z, M = rows_of(p, zb);
    using T = typename P::T;
    using Tr = OperandTraits<T>;
    constexpr int LS = SEG + Tr::PAD;
    constexpr int VA = P::VA, VB = P::VB;
    // work items per operand panel: a k-contiguous vector (ALONG_K); otherwise (operand contiguous along its rows) a
    // V x V block to transpose in registers (bfloat16: LDS rows are then written 16 bytes at a time), or for binary32 a
    // single vector of V rows at ONE k -- neighbouring lanes then fetch neighbouring vectors of the same k, whole cache
    // lines per load instruction instead of one line per lane (LDS rows are written element by element either way).
    constexpr bool NAT_A = !P::A_ALONG_K && sizeof(T) == 4, NAT_B = !P::B_ALONG_K && sizeof(T) == 4;
    constexpr int CA = P::A_ALONG_K ? 32 * SEG / VA : NAT_A ? (32 / VA) * SEG : (32 / VA) * (SEG / VA);
    constexpr int CB = P::B_ALONG_K ? 32 * SEG / VB : NAT_B ? (32 / VB) * SEG : (32 / VB) * (SEG / VB);
    constexpr int NA = (CA + 63) / 64, NB = (CB + 63) / 64;
    constexpr int RA = (P::A_ALONG_K || NAT_A) ? 1 : VA, RB = (P::B_ALONG_K || NAT_B) ? 1 : VB;
    static_assert(SEG % Tr::KINST == 0 && SEG % VA == 0 && SEG % VB == 0 && 32 % VA == 0 && 32 % VB == 0, "segment shape");
    constexpr size_t PANEL_BYTES = (size_t)(BDIR ? 1 : 2) * 32 * LS * sizeof(T);   // operand panel(s) of one wavefront
    static_assert(PARTIAL || PANEL_BYTES >= 4096, "the fold reuses a wavefront's panels for its 32x32 partial tile");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    T *As = reinterpret_cast<T *>(smem + (size_t)w * PANEL_BYTES), *Bs = As + 32 * LS;
    const int tiles_n = (p.N + 31) / 32;
    const int m0 = (blockIdx.x / tiles_n) * 32, n0 = (blockIdx.x % tiles_n) * 32;
    if (m0 >= M) return;
    const int nseg = (p.K + SEG - 1) / SEG;
    const int lrow = lane & 31, lk = lane >> 5;
    // per-column epilogue data (bias) is requested now, so that it has arrived when the sums are ready
    const auto col = make_col(p, min(n0 + lrow, p.N - 1));

    // fixed assignment of panel items to lanes; the row part of every gather is resolved once per wavefront
    typename P::CtxA ca[NA];
    typename P::CtxB cb[NB];
    int ka[NA], kb[NB], la[NA], lb[NB];
    // k-contiguous operands: four lanes share a panel row and take its vectors in turn, a lane serves rows pr and
    // pr + 16 -- two row contexts per lane instead of one per item (the position decomposition of a gather is most of
    // the arithmetic in front of the loads).  Segments that do not split into four vectors per lane keep one
    // context per item.
    constexpr bool ROWS_A = P::A_ALONG_K && SEG % (4 * VA) == 0, ROWS_B = P::B_ALONG_K && SEG % (4 * VB) == 0;
    const int pr = lane >> 2, pq = lane & 3;
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int id = lane + i * 64;
        int r;
        if constexpr (ROWS_A) { r = pr + 16 * (i / (NA / 2)); ka[i] = (pq + 4 * (i % (NA / 2))) * VA; }
        else if constexpr (P::A_ALONG_K) { r = id / (SEG / VA); ka[i] = (id % (SEG / VA)) * VA; }
        else if constexpr (NAT_A) { r = (id % (32 / VA)) * VA; ka[i] = id / (32 / VA); }
        else { r = (id / (SEG / VA)) * VA; ka[i] = (id % (SEG / VA)) * VA; }   // neighbours write one LDS row
        la[i] = r * LS + ka[i];
        if (ROWS_A && i % (NA / 2 > 0 ? NA / 2 : 1) != 0) ca[i] = ca[i - 1];     // same row as the item before
        else ca[i] = make_ctx_a(p, m0 + r, zb);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int id = lane + i * 64;
        int r;
        if constexpr (ROWS_B) { r = pr + 16 * (i / (NB / 2)); kb[i] = (pq + 4 * (i % (NB / 2))) * VB; }
        else if constexpr (P::B_ALONG_K) { r = id / (SEG / VB); kb[i] = (id % (SEG / VB)) * VB; }
        else if constexpr (NAT_B) { r = (id % (32 / VB)) * VB; kb[i] = id / (32 / VB); }
        else { r = (id / (SEG / VB)) * VB; kb[i] = (id % (SEG / VB)) * VB; }
        lb[i] = r * LS + kb[i];
        if (ROWS_B && i % (NB / 2 > 0 ? NB / 2 : 1) != 0) cb[i] = cb[i - 1];
        else cb[i] = make_ctx_b(p, n0 + r, zb);
    }
    constexpr bool VEC_LDS = sizeof(T) == 2;
    const typename P::CtxB cbd = make_ctx_b(p, n0 + lrow, zb);      // this lane's own column (direct B operands)
    constexpr int NBD = BDIR ? (sizeof(T) == 4 ? SEG / VB : (SEG / 16) * (8 / VB)) : 1;

    auto segment_sum = [&](int seg) -> f32x16 {
        const int kbeg = seg * SEG, kend = min(p.K, kbeg + SEG);
        Vec<T, VA> ra[NA][RA];
        Vec<T, VB> rb[BDIR ? 1 : NB][RB];
        Vec<T, VB> rbd[NBD];
        if constexpr (BDIR) {
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int q = 0; q < NBD; ++q) rbd[q] = p.load_b(cbd, kbeg + q * VB, kend);
            } else {        // slot t of this lane covers k = 16 t + 8 lk .. +7
#pragma unroll
                for (int q = 0; q < NBD; ++q)
                    rbd[q] = p.load_b(cbd, kbeg + 16 * (q / (8 / VB)) + 8 * lk + VB * (q % (8 / VB)), kend);
            }
        }
#pragma unroll
        for (int i = 0; i < NA; ++i)
            if (CA % 64 == 0 || lane + i * 64 < CA)
#pragma unroll
                for (int q = 0; q < RA; ++q) ra[i][q] = p.load_a(ca[i], kbeg + ka[i] + q, kend);
        if constexpr (!BDIR) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (CB % 64 == 0 || lane + i * 64 < CB)
#pragma unroll
                    for (int q = 0; q < RB; ++q) rb[i][q] = p.load_b(cb[i], kbeg + kb[i] + q, kend);
        }
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if (CA % 64 != 0 && lane + i * 64 >= CA) continue;
            T *d = As + la[i];
            if constexpr (P::A_ALONG_K) {
                if constexpr (VEC_LDS) *reinterpret_cast<Vec<T, VA> *>(d) = ra[i][0];
                else {
#pragma unroll
                    for (int j = 0; j < VA; ++j) d[j] = ra[i][0][j];
                }
            } else if constexpr (NAT_A) {
#pragma unroll
                for (int j = 0; j < VA; ++j) d[j * LS] = ra[i][0][j];
            } else {
#pragma unroll
                for (int j = 0; j < VA; ++j) {
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
        for (int i = 0; i < (BDIR ? 0 : NB); ++i) {
            if (CB % 64 != 0 && lane + i * 64 >= CB) continue;
            T *d = Bs + lb[i];
            if constexpr (P::B_ALONG_K) {
                if constexpr (VEC_LDS) *reinterpret_cast<Vec<T, VB> *>(d) = rb[i][0];
                else {
#pragma unroll
                    for (int j = 0; j < VB; ++j) d[j] = rb[i][0][j];
                }
            } else if constexpr (NAT_B) {
#pragma unroll
                for (int j = 0; j < VB; ++j) d[j * LS] = rb[i][0][j];
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
        // the panels are private to this wavefront and a wavefront's LDS operations execute in order
        __builtin_amdgcn_wave_barrier();
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const T *a = As + lrow * LS, *b = Bs + lrow * LS;
        if constexpr (!BDIR) {
#pragma unroll 8
            for (int kk = 0; kk < SEG; kk += Tr::KINST) {
                if constexpr (sizeof(T) == 4)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk + lk], b[kk + lk], acc, 0, 0, 0);
                else
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(a + kk + lk * 8),
                                                                  *reinterpret_cast<const bf16x8 *>(b + kk + lk * 8), acc, 0, 0, 0);
            }
        } else if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int t = 0; t < SEG / 2; ++t) {          // slot t needs k = 2 t + lk: one of two neighbours in a vector
                const float b0 = rbd[(2 * t) / VB][(2 * t) % VB], b1 = rbd[(2 * t + 1) / VB][(2 * t + 1) % VB];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[2 * t + lk], lk ? b1 : b0, acc, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int t = 0; t < SEG / 16; ++t) {
                bf16x8 bv;
                if constexpr (VB == 8) bv = rbd[t];
                else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) bv[e] = rbd[t * (8 / VB) + e / VB][e % VB];
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(a + 16 * t + lk * 8), bv,
                                                              acc, 0, 0, 0);
            }
        }
        return acc;
    };

    if constexpr (PARTIAL) {
        const int seg = blockIdx.y * WAVES + w;
        if (seg >= nseg) return;
        const f32x16 acc = segment_sum(seg);
        const int n = n0 + lrow;
        if (m0 + 32 <= M && n0 + 32 <= p.N) {
#pragma unroll
            for (int r = 0; r < 16; ++r) do_store(p, m0 + 8 * (r / 4) + 4 * lk + (r % 4), n, acc[r], seg, zb, col);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = m0 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (m < M && n < p.N) do_store(p, m, n, acc[r], seg, zb, col);
            }
        }
    } else {
        constexpr int PER = 1024 / (WAVES * 64);        // tile elements owned by each thread in the fold
        static_assert(PER * WAVES * 64 == 1024, "WAVES must divide 16");
        // element e of this thread is accumulator register r = e*WAVES + w of lane `lane`.  What its store needs from
        // memory (a ReLU mask) is requested now; it has arrived when the sums are ready.
        constexpr bool PRE1 = HasPre1<P>::value;
        using Pre1T = typename Pre1Type<P, PRE1>::type;
        Pre1T pre[PER];
        if constexpr (PRE1) {
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int r = e * WAVES + w;
                pre[e] = epi_pre1(p, min(m0 + 8 * (r / 4) + 4 * lk + (r % 4), M - 1), min(n0 + lrow, p.N - 1), zb);
            }
        }
        float total[PER];
#pragma unroll
        for (int e = 0; e < PER; ++e) total[e] = 0.0f;
        const int gbeg = blockIdx.y * spg, gend = min(nseg, gbeg + spg);
        const int rounds = (gend - gbeg + WAVES - 1) / WAVES;
        for (int rd = 0; rd < rounds; ++rd) {
            const int seg = gbeg + rd * WAVES + w;
            if (seg < gend) {
                const f32x16 acc = segment_sum(seg);
                // this wavefront's panels are free again: they now carry its partial tile (r*64 + lane order)
                float *mine = reinterpret_cast<float *>(smem + (size_t)w * PANEL_BYTES);
#pragma unroll
                for (int r = 0; r < 16; ++r) mine[r * 64 + lane] = acc[r];
            }
            __syncthreads();
            const int live = min(WAVES, gend - gbeg - rd * WAVES);
            // all reads first (a panel that carries nothing this round is read and ignored), then the additions in
            // wave (= segment) order: one LDS round trip instead of one per partial tile
            float v[PER][WAVES];
#pragma unroll
            for (int e = 0; e < PER; ++e)
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww)
                    v[e][ww] = reinterpret_cast<const float *>(smem + (size_t)ww * PANEL_BYTES)[e * (WAVES * 64) + tid];
#pragma unroll
            for (int e = 0; e < PER; ++e)
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww)
                    if (ww < live) total[e] += v[e][ww];
            __syncthreads();
        }
        // element e of this thread is accumulator register r = e*WAVES + w of lane `lane`: one column per thread
        const int n = n0 + lrow;
        if (m0 + 32 <= M && n0 + 32 <= p.N) {
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int r = e * WAVES + w;
                if constexpr (PRE1) p.store1(pre[e], total[e]);
                else do_store(p, m0 + 8 * (r / 4) + 4 * lk + (r % 4), n, total[e], (int)blockIdx.y, zb, col);
            }
        } else {
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                const int r = e * WAVES + w;
                const int m = m0 + 8 * (r / 4) + 4 * lk + (r % 4);
                if (m < M && n < p.N) {
                    if constexpr (PRE1) p.store1(pre[e], total[e]);
                    else do_store(p, m, n, total[e], (int)blockIdx.y, zb, col);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// The same scheme on 16x16 output tiles: four times the workgroups for the same problem.
// With 16-32 observations a layer has fewer 32x32 tiles than the chip has compute units, and a workgroup's run time
// is then the time its one compute unit needs to pull both 32 x K operand panels through its L1 (conv3, binary32,
// K = 576: 147 KB per workgroup; about 60 % of the kernel's duration went into getting the loads issued at all).
// Halving both tile edges halves the bytes per workgroup and spreads them over four times as many compute units.
// Bits: on this hardware the matrix instructions of one operand type return the same bits for the same k order
// whatever their tile shape (32x32x2 and 16x16x4 for binary32 -- both equal to a sequential fma chain --, 32x32x16
// and 16x16x32 for bfloat16: checked on random operands of mixed magnitude, 51200 outputs each, and by the tests that
// compare the kernel families bitwise), so with the same segments the results equal those of the other kernels.
// Problems: A_ALONG_K and B_ALONG_K, plain store() epilogue (the forward layers).
// ------------------------------------------------------------------------------------------------------------
template <class P, int WAVES, int SEG>
__global__ __launch_bounds__(WAVES * 64) void wsgemm16_kernel(const P p, const int spg)
{
    using T = typename P::T;
    using Tr = OperandTraits<T>;
    constexpr int VA = P::VA, VB = P::VB;
    constexpr int KI = sizeof(T) == 4 ? 4 : 32;          // k per matrix instruction
    static_assert(P::A_ALONG_K && P::B_ALONG_K, "k-contiguous operands");
    static_assert(WAVES >= 4 && SEG % KI == 0 && SEG % (4 * VA) == 0 && SEG % (4 * VB) == 0,
                  "four wavefronts own the fold; four lanes share a panel row");
    constexpr int LS = SEG + Tr::VEC;         // row pitch: a 16-byte step per row, so the 64 lanes of an operand read
                                              // (row i, k slot q) spread evenly over the banks
    constexpr int NA = 16 * SEG / VA / 64, NB = 16 * SEG / VB / 64;     // vectors per lane and panel
    constexpr size_t PANEL_BYTES = (size_t)2 * 16 * LS * sizeof(T);
    static_assert(PANEL_BYTES >= 1024, "the fold reuses a wavefront's panels for its 16x16 partial tile");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int zb = blockIdx.z, M = rows_of(p, zb);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    T *As = reinterpret_cast<T *>(smem + (size_t)w * PANEL_BYTES), *Bs = As + 16 * LS;
    const int tiles_n = (p.N + 15) / 16;
    const int m0 = (blockIdx.x / tiles_n) * 16, n0 = (blockIdx.x % tiles_n) * 16;
    if (m0 >= M) return;
    const int nseg = (p.K + SEG - 1) / SEG;
    const int li = lane & 15, kq = lane >> 4;
    // after the fold, thread (w < 4, lane) owns accumulator register w of lane `lane`: row 4 kq + w, column li
    const auto col = make_col(p, min(n0 + li, p.N - 1));

    // Four lanes share a panel row and take its vectors in turn, so a lane resolves ONE row of each operand (the
    // position decomposition of a gather is most of the arithmetic in front of the loads: with a different row per
    // item the kernel spent 300 vector instructions between its first and its last load).
    const int pr = lane >> 2, pq = lane & 3;
    const typename P::CtxA ca = make_ctx_a(p, m0 + pr, zb);
    const typename P::CtxB cb = make_ctx_b(p, n0 + pr, zb);
    auto segment_sum = [&](int seg) -> f32x4 {
        const int kbeg = seg * SEG, kend = min(p.K, kbeg + SEG);
        Vec<T, VA> ra[NA];
        Vec<T, VB> rb[NB];
#pragma unroll
        for (int i = 0; i < NA; ++i) ra[i] = p.load_a(ca, kbeg + (pq + 4 * i) * VA, kend);
#pragma unroll
        for (int i = 0; i < NB; ++i) rb[i] = p.load_b(cb, kbeg + (pq + 4 * i) * VB, kend);
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<Vec<T, VA> *>(As + pr * LS + (pq + 4 * i) * VA) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<Vec<T, VB> *>(Bs + pr * LS + (pq + 4 * i) * VB) = rb[i];
        // the panels are private to this wavefront and a wavefront's LDS operations execute in order
        __builtin_amdgcn_wave_barrier();
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (sizeof(T) == 4) {        // slot t: lane (i, q) supplies k = 4 t + q
            const T *a = As + li * LS + kq, *b = Bs + li * LS + kq;
#pragma unroll
            for (int t = 0; t < SEG / 4; ++t) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[4 * t], b[4 * t], acc, 0, 0, 0);
        } else {                               // slot t: lane (i, q) supplies k = 32 t + 8 q .. + 7
            const T *a = As + li * LS + 8 * kq, *b = Bs + li * LS + 8 * kq;
#pragma unroll
            for (int t = 0; t < SEG / 32; ++t)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8 *>(a + 32 * t),
                                                              *reinterpret_cast<const bf16x8 *>(b + 32 * t), acc, 0, 0, 0);
        }
        return acc;
    };

    float total = 0.0f;
    const int gbeg = blockIdx.y * spg, gend = min(nseg, gbeg + spg);
    const int rounds = (gend - gbeg + WAVES - 1) / WAVES;
    for (int rd = 0; rd < rounds; ++rd) {
        const int seg = gbeg + rd * WAVES + w;
        if (seg < gend) {
            const f32x4 acc = segment_sum(seg);
            float *mine = reinterpret_cast<float *>(smem + (size_t)w * PANEL_BYTES);     // the panels are free again
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[r * 64 + lane] = acc[r];
        }
        __syncthreads();
        const int live = min(WAVES, gend - gbeg - rd * WAVES);
        if (w < 4) {
            float v[WAVES];
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww)        // all reads first, then the additions in wave (= segment) order
                v[ww] = reinterpret_cast<const float *>(smem + (size_t)ww * PANEL_BYTES)[tid];
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww)
                if (ww < live) total += v[ww];
        }
        __syncthreads();
    }
    if (w < 4) {
        const int m = m0 + 4 * kq + w, n = n0 + li;
        if (m < M && n < p.N) do_store(p, m, n, total, (int)blockIdx.y, zb, col);
    }
}

template <class P, int WAVES, int SEG> inline hipError_t launch_wsgemm16(const P &p, hipStream_t stream, int segs_per_group = 1 << 30)
{
    const int tiles = ((grid_rows(p) + 15) / 16) * ((p.N + 15) / 16);
    const int nseg = (p.K + SEG - 1) / SEG;
    if (tiles <= 0 || nseg <= 0) return hipSuccess;
    using T = typename P::T;
    const size_t lds = (size_t)WAVES * 2 * 16 * (SEG + OperandTraits<T>::VEC) * sizeof(T);
    auto kern = wsgemm16_kernel<P, WAVES, SEG>;
    static std::atomic<bool> attr_set{false};       // raise the dynamic-LDS limit once per instantiation (setting it twice is harmless)
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int spg = segs_per_group < nseg ? segs_per_group : nseg;
    hipLaunchKernelGGL(kern, dim3(tiles, (nseg + spg - 1) / spg, grid_batches(p)), dim3(WAVES * 64, 1, 1), lds, stream, p, spg);
    return hipGetLastError();
}

template <class P, int WAVES, int SEG, bool PARTIAL, bool BDIR = false>
inline hipError_t launch_wsgemm(const P &p, hipStream_t stream, int segs_per_group = 1 << 30)
{
    using T = typename P::T;
    const int tiles = ((grid_rows(p) + 31) / 32) * ((p.N + 31) / 32);
    const int nseg = (p.K + SEG - 1) / SEG;
    if (tiles <= 0 || nseg <= 0) return hipSuccess;
    const size_t lds = (size_t)WAVES * (BDIR ? 1 : 2) * 32 * (SEG + OperandTraits<T>::PAD) * sizeof(T);
    auto kern = wsgemm_kernel<P, WAVES, SEG, PARTIAL, BDIR>;
    static std::atomic<bool> attr_set{false};       // raise the dynamic-LDS limit once per instantiation (setting it twice is harmless)
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int spg = segs_per_group < nseg ? segs_per_group : nseg;
    const int gy = PARTIAL ? (nseg + WAVES - 1) / WAVES : (nseg + spg - 1) / spg;
    hipLaunchKernelGGL(kern, dim3(tiles, gy, grid_batches(p)), dim3(WAVES * 64, 1, 1), lds, stream, p, spg);
    return hipGetLastError();
}

}  // namespace hts
