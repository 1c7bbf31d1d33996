// bf16 MFMA GEMM of the frozen base weight with the per-segment adapter fused in.
//
//   forward  (NN = false):  C[m][n] = sum_k Aop[m][k] * Bop[n][k]   (Bop = W [d_out][d_in], K-contiguous)
//   backward (NN = true) :  C[m][n] = sum_k Aop[m][k] * Bop[k][n]   (Bop = W [d_out][d_in], N-contiguous)
//
// plus, for every LoRA segment that meets the row tile, extra K-steps
//   forward : C += Hs[m][p] * B_i[n][p]      (Hs = s_i * X A_i^T from the shrink kernel)
//   backward: C += dH[m][p] * A_i[p][n]      (dH = s_i * dY B_i)
// where Hs / dH arrive as a bf16 value plus a bf16 rounding residual (two 16-wide rank blocks per
// 32-wide K-step), accumulated in the same fp32 accumulators before the single rounding to bf16,
// and an epilogue with the optional bias, the optional store of the pre-adapter output, the IA3
// per-channel scale of each row's own segment and the privacy flow's noise effect.
//
// One kernel on v_mfma_f32_16x16x32_bf16: 4 wavefronts (2x2), each NBLK x NBLK blocks of 16x16 of C.
// NBLK = 8: 256x256 tile of the workgroup, all 256 accumulation registers per wavefront, 160 KiB of
// LDS, for launches with enough such tiles to fill the chip.  NBLK = 4: 128x128 tile, 64 accumulation
// registers, 80 KiB of LDS, two workgroups per CU, for everything smaller.  The text below describes
// the 256x256 case; the 128x128 one is the same code with half the extents.  Why this instruction:
// with Gaussian operands the power-limited chip sustains about 12 % more flops on the 16x16x32 form
// than on the 32x32x16 form.
//
// A wavefront's 128x128 of C is 8x8 blocks of 16x16, 4 registers each: all 256 accumulation
// registers.  They are not C++ objects: every piece of code that touches one is an assembly
// template that names a0..a255 literally (gemm16_asm.hpp; block (i, j) is a[4(8i+j) .. +3]), and
// the compiler-generated code between the templates must not use accumulation registers for
// anything (a CPU test inspects the generated assembly for that).  The MFMA is issued as (weight
// fragment, activation fragment): a lane ends up with C[16i + l%16][16j + 4(l/16) + 0..3], i.e. runs
// of 4 consecutive n of one row m: rows keep their own segment in the epilogue, which stages the
// bf16 tile through LDS and writes whole rows.
#pragma once
#include <type_traits>

#include "gemm16_asm.hpp"
#include "symb_device.hpp"

namespace symb {

struct GemmParams {
    const bf16* Aop;            // [M][K] (null when the rows come from per-segment buffers, see a_seg)
    const bf16* Bop;            // NT: [N][K]   NN: [K][N]
    bf16* C;                    // [M][N]
    bf16* Cbase;                // [M][N] or null: accumulator (+bias) before the adapter term
    const bf16* bias;           // [N] or null
    int M, N, K;
    int num_m_tiles, num_n_tiles, group_m;
    const int32_t* off;         // device [S+1]
    const SegDesc* seg;         // device [S]
    const int32_t* tile_seg_lo; // device [num_m_tiles]: first / last non-empty segment meeting the row tile
    const int32_t* tile_seg_hi;
    const bf16* ext;            // [M][ext_pitch] bf16: Hs (forward) or dH (backward), per row rpad values
                                // then rpad residuals of the row's own segment; null = no LoRA term
    int ext_pitch;
    int epi_ia3;                // 0, or the adapter kind whose rows the epilogue scales by its vector l_i[n]
    const int32_t* tile_epi;    // with epi_ia3: per row tile, 1 if it holds rows of such a segment (the others take the plain epilogue)
                                // (IA3 in the forward, IA3_IN in the input gradient)
    // Per-segment buffers instead of flat tensors (device arrays of S pointers, or null): row t of
    // segment i is a_seg[i] + (t - off[i]) * K resp. c_seg[i] + (t - off[i]) * N.  All a_seg buffers lie
    // within 4 GiB above a_base (checked by the host), so lane offsets from a_base fit 32 bits.
    const bf16* const* a_seg;
    const bf16* a_base;
    bf16* const* c_seg;
    const NoiseDesc* neff;      // device [S] or null: per-segment noise effect subtracted last (privacy flow)
    // K-split (k_parts <= 1: off): of every XCD's run of tiles, those from number k_whole on are computed
    // by k_parts workgroups each; partial holds k_parts fp32 tiles per split tile, k_count one zeroed
    // arrival counter per split tile.
    int k_parts, k_whole;
    float* partial;
    int* k_count;
    double timing_flops;        // host bookkeeping for the measurement hook; unused on the device
};

// 16-byte chunk swizzle of a K-contiguous tile row (8 chunks of 8 bf16 per row).
__device__ __forceinline__ int swz_row(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// K-contiguous tile: [rows][64] bf16, 128 B per row, chunk kc stored at kc ^ swz_row(row).
__device__ __forceinline__ int lds_off_kmajor(int row, int kc) { return row * 128 + ((kc ^ swz_row(row)) << 4); }

__device__ __forceinline__ uint4 ld_global_16(const bf16* p, bool ok) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (ok) v = *reinterpret_cast<const uint4*>(p);
    return v;
}

template <int NBLK>
struct Gemm16Tile {
    static_assert(NBLK == 8 || NBLK == 4, "256x256 or 128x128 tile");
    static constexpr int BM = 32 * NBLK, BN = 32 * NBLK, NT = 256, BK = 64;
    static constexpr int WT = 16 * NBLK;                 // rows and columns of a wavefront's part
    static constexpr int UNIT = BM * 128;                // one operand's 64-k stage
    static constexpr int C_PITCH = BN * 2 + 16, C_BYTES = BM * C_PITCH;
    static constexpr int SMEM = 5 * UNIT;                // three A units, two B units
    static_assert(C_BYTES <= SMEM, "the staged output tile must fit the ring");
};

// N-contiguous weight unit: [64 k][BN n] bf16, 16-byte chunk nc of row k stored at nc ^ swz.  The
// transposing read of one 16-lane group fetches 4 k-rows x 32 B: the (k & 3) term lays those side
// by side (128 B), the (k >> 2) term moves the next group (4 k-rows further) to the other half of
// the banks.
__device__ __forceinline__ int swz_nmajor16(int k) { return ((k & 3) << 1) ^ (((k >> 2) & 1) << 3); }
template <int BN>
__device__ __forceinline__ int lds_off_nmajor16(int k, int nc) { return k * (BN * 2) + ((nc ^ swz_nmajor16(k)) << 4); }

template <int I0, int I1, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I0 < I1) {
        f(std::integral_constant<int, I0>{});
        static_for<I0 + 1, I1>(f);
    }
}

// The four accumulators of block R / 4 of this lane.
template <int R>
__device__ __forceinline__ void acc16_read4(float& v0, float& v1, float& v2, float& v3) {
    asm volatile("v_accvgpr_read_b32 %0, a[%4]\n\tv_accvgpr_read_b32 %1, a[%5]\n\t"
                 "v_accvgpr_read_b32 %2, a[%6]\n\tv_accvgpr_read_b32 %3, a[%7]"
                 : "=v"(v0), "=v"(v1), "=v"(v2), "=v"(v3)
                 : "n"(R), "n"(R + 1), "n"(R + 2), "n"(R + 3));
}

template <int R>
__device__ __forceinline__ void acc16_write4(float v0, float v1, float v2, float v3) {
    asm volatile("v_accvgpr_write_b32 a[%4], %0\n\tv_accvgpr_write_b32 a[%5], %1\n\t"
                 "v_accvgpr_write_b32 a[%6], %2\n\tv_accvgpr_write_b32 a[%7], %3"
                 :
                 : "v"(v0), "v"(v1), "v"(v2), "v"(v3), "n"(R), "n"(R + 1), "n"(R + 2), "n"(R + 3));
}

// PLAIN: no bias, no IA3 scale, no noise effect, no pre-adapter output (checked by the host).
template <int NBLK, bool NN, bool PLAIN>
__global__ void __launch_bounds__(256)
symb_gemm16_kernel(const GemmParams p) {
    using TT = Gemm16Tile<NBLK>;
    constexpr int BM = TT::BM, BN = TT::BN, NT = TT::NT, CP = TT::C_PITCH, WT = TT::WT;
    constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;      // 16-byte chunks per thread of a register-staged tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* const sA = smem;                        // register-staged tiles (K remainder, LoRA term)
    unsigned char* const sB = smem + TT::UNIT;

    // ---- tile of this workgroup
    // Every XCD (blockIdx & 7) walks a contiguous run of per_xcd tiles.  With a K-split (k_parts > 1)
    // the tiles of that run from number k_whole on are computed by k_parts workgroups each, one per
    // K range, all on this XCD: all tiles of a launch too small to fill the chip
    // (k_whole = 0), or the tiles of a last, mostly empty round.
    const int total = p.num_m_tiles * p.num_n_tiles;
    int lin, part = 0, nparts = 1, slot = 0;
    {
        const int per_xcd = (total + 7) >> 3;
        const int item = blockIdx.x >> 3;
        int li = item;
        if (p.k_parts > 1 && item >= p.k_whole) {
            // part-major: first every split tile's last K range (the one that also has the K remainder
            // to do), then the one before ...: tiles that run side by side then walk
            // the same K range and share their operand panels in L2
            const int j = item - p.k_whole, nsplit = per_xcd - p.k_whole;
            nparts = p.k_parts;
            part = nparts - 1 - j / nsplit;
            li = p.k_whole + j % nsplit;
            slot = (blockIdx.x & 7) * nsplit + (li - p.k_whole);   // partial tiles and counter of this tile
        }
        lin = (blockIdx.x & 7) * per_xcd + li;
        if (lin >= total || li >= per_xcd) return;
    }
    const int width = p.group_m * p.num_n_tiles;
    const int first_m = (lin / width) * p.group_m;
    const int gsz = min(p.num_m_tiles - first_m, p.group_m);
    const int tm = first_m + (lin % width) % gsz;
    const int tn = (lin % width) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * WT, wn0 = (wave & 1) * WT;
    const int l15 = lane & 15, lg = lane >> 4;
    const int seg_lo = p.tile_seg_lo[tm], seg_hi = p.tile_seg_hi[tm];
    auto a_row = [&](int m) __attribute__((always_inline)) -> const bf16* {
        if (!p.a_seg) return p.Aop + (size_t)m * p.K;
        const int s = seg_of_row(p.off, seg_lo, seg_hi, m);
        return p.a_seg[s] + (size_t)(m - p.off[s]) * p.K;
    };
    const bf16* const a_tile = p.a_seg ? p.a_base : p.Aop + (size_t)m0 * p.K;
    const bf16* const b_tile = NN ? (p.Bop + n0) : (p.Bop + (size_t)n0 * p.K);
    const unsigned lds0 = (unsigned)(size_t)smem;          // LDS byte address of the dynamic segment

    // ---- register-staged 64-k tile (K remainder, LoRA term).  Chunk i of a thread sits 32 rows
    // (K-contiguous tiles) or KSTEP k-rows (N-contiguous weight tile) below chunk 0.
    constexpr int RSTEP = NT / 8, KSTEP = NT / (BN / 8);
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;
    const int nn_k = tid / (BN / 8), nn_nc = tid % (BN / 8);
    const int a_lds0 = lds_off_kmajor(lrow, tid & 7);
    const int b_lds0 = NN ? lds_off_nmajor16<BN>(nn_k, nn_nc) : a_lds0;
    uint4 ra[CA], rb[CB];
    auto lds_store_a = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < CA; ++i) *reinterpret_cast<uint4*>(sA + a_lds0 + i * RSTEP * 128) = ra[i];
    };
    auto lds_store_b = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            if constexpr (!NN) *reinterpret_cast<uint4*>(sB + b_lds0 + i * RSTEP * 128) = rb[i];
            else *reinterpret_cast<uint4*>(sB + b_lds0 + i * KSTEP * (BN * 2)) = rb[i];
        }
    };
    auto gload_tail = [&](int k0) __attribute__((always_inline)) {
        const bool kok = (k0 + lkc) < p.K;
#pragma unroll
        for (int i = 0; i < CA; ++i)
            ra[i] = ld_global_16(a_row(min(m0 + lrow + i * RSTEP, p.M - 1)) + k0 + lkc, kok);
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            if constexpr (!NN)
                rb[i] = ld_global_16(p.Bop + (size_t)min(n0 + lrow + i * RSTEP, p.N - 1) * p.K + k0 + lkc, kok);
            else {
                const int kr = k0 + nn_k + i * KSTEP;
                rb[i] = ld_global_16(p.Bop + (size_t)min(kr, p.K - 1) * p.N + n0 + min(nn_nc * 8, p.N - 8 - n0), kr < p.K);
            }
        }
    };
    // ---- LoRA term, first part: its k-steps are 32 wide (value half and residual half of a rank
    // block of 16), staged through registers, 4 chunks of 16 bytes per thread and operand.  A step is
    // (segment es, first extended column ekc); ext_seek moves es to the next LoRA segment with rows
    // in this tile, ext_load fetches the step.  The first step is fetched here, so that its latency
    // hides under the main loop.
    constexpr int EC = BM / 64;                              // 16-byte chunks per thread of a 32-k tile
    // K-contiguous 32-k tile: chunk i sits 64 rows below chunk 0.  Steps alternate between the two 32-k
    // halves of the 64-k tile, so a step's stores never meet the reads of the step before it.
    const int e_lds[2] = {lds_off_kmajor(tid >> 2, tid & 3), lds_off_kmajor(tid >> 2, 4 + (tid & 3))};
    constexpr int ESETS = (NN ? 1 : 2) + (NBLK == 8 ? 0 : 1);  // steps in flight (register sets): what fits without spilling
    uint4 ea[ESETS][EC], eb[ESETS][EC];
    int e_rlo[ESETS] = {}, e_rhi[ESETS] = {};                // the rows of the segment of the step in each set
    bool e_have[ESETS] = {};                                 // the set holds a step that has not run yet
    int es = seg_lo, ekc = 0, e_lo = 0, e_hi = 0;
    bool ext_more = false;                                   // a further step exists at (es, ekc)
    SegDesc esd;
    auto ext_seek = [&]() __attribute__((always_inline)) -> bool {
        for (; es <= seg_hi; ++es) {
            esd = p.seg[es];
            e_lo = max(p.off[es], m0);
            e_hi = min(min(p.off[es + 1], m0 + BM), p.M);
            if (esd.kind == KIND_LORA && e_hi > e_lo) return true;      // uniform over the workgroup
        }
        return false;
    };
    // The parts of a K-split 128x128 tile share the tile's steps out: step number e_no (counted over the
    // tile) belongs to part e_no % nparts.  Any part may take any step, the partial tiles are added up
    // anyway; left to the last part alone, a tile of many short segments had its steps one after the
    // other behind that part's share of K while the other parts were done (a call of 128 rows in 16
    // segments: 43.6 -> 34.2 us).  The split last round of 256x256 tiles keeps them with the last part
    // (sharing them out there measured 0.4 % slower on the mixed workload).
    int e_no = 0;
    auto ext_next = [&]() __attribute__((always_inline)) {
        ekc += 32;
        ++e_no;
        if (ekc >= 2 * esd.rpad) {
            ++es;
            ekc = 0;
            ext_more = ext_seek();
        }
    };
    auto ext_skip = [&]() __attribute__((always_inline)) {
        if (nparts > 1)
            while (ext_more && (NBLK == 8 ? nparts - 1 : e_no % nparts) != part) ext_next();
    };
    // Fetches the step at (es, ekc) into register set SET and moves on to this part's next step.
    auto ext_load = [&](auto SETC) __attribute__((always_inline)) {
        constexpr int SET = decltype(SETC)::value;
        // activation-side tile: rows of this segment only, others zero
#pragma unroll
        for (int i = 0; i < EC; ++i) {
            const int m = m0 + (tid >> 2) + i * 64;
            const bool ok = m >= e_lo && m < e_hi;
            ea[SET][i] = ld_global_16(p.ext + (size_t)(ok ? m : 0) * p.ext_pitch + ekc + (tid & 3) * 8, ok);
        }
        // adapter-side tile; both halves of the extended columns meet the same adapter matrix
#pragma unroll
        for (int i = 0; i < EC; ++i) {
            if constexpr (!NN) {       // B_i [N][rank], rank-contiguous
                const int n = n0 + (tid >> 2) + i * 64;
                const int pk = ekc + (tid & 3) * 8, pp = pk >= esd.rpad ? pk - esd.rpad : pk;
                uint4 v = make_uint4(0u, 0u, 0u, 0u);
                if (n < p.N && pp < esd.rank) {
                    const bf16* src = esd.B + (size_t)n * esd.rank + pp;
                    if ((esd.rank & 7) == 0) {
                        v = *reinterpret_cast<const uint4*>(src);
                    } else {
                        unsigned short e[8];
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            e[q] = (pp + q < esd.rank) ? reinterpret_cast<const unsigned short*>(src)[q] : (unsigned short)0;
                        v.x = e[0] | ((unsigned)e[1] << 16); v.y = e[2] | ((unsigned)e[3] << 16);
                        v.z = e[4] | ((unsigned)e[5] << 16); v.w = e[6] | ((unsigned)e[7] << 16);
                    }
                }
                eb[SET][i] = v;
            } else {                   // A_i [rank][N], N-contiguous
                const int n = n0 + nn_nc * 8;
                const int pk = ekc + nn_k + i * KSTEP, pp = pk >= esd.rpad ? pk - esd.rpad : pk;
                const bool ok = pp < esd.rank && n < p.N;
                eb[SET][i] = ld_global_16(esd.A + (size_t)(ok ? pp : 0) * p.N + (ok ? n : 0), ok);
            }
        }
        e_rlo[SET] = e_lo;
        e_rhi[SET] = e_hi;
        ext_next();
        ext_skip();
    };
    const bool last_part = part == nparts - 1;      // the K remainder goes with the last K range
    ext_more = p.ext != nullptr && ext_seek();
    ext_skip();
    e_have[0] = ext_more;
    if (e_have[0]) ext_load(std::integral_constant<int, 0>{});


    // Lane byte offsets of the MFMA fragments of 32-k step ks inside an operand's 64-k tile.  Lane
    // group g = l/16 holds row l%16 and k = 32 ks + 16 q + 8 (g/2) + 4 (g%2) + 0..3, q = 0, 1 (one
    // 8-byte read each: half g%2 of 16-byte chunk 4 ks + 2 q + g/2).  For the N-contiguous weight one
    // address per 16-column block j serves both reads (the transposing read: lane jj of a 16-lane
    // group fetches k-row jj/4, columns 4 (jj%4) .. +3, and receives column jj of 4 k-rows; the
    // second read, 16 k-rows down, is a constant offset away).
    auto frag_a = [&](int ks, int q) __attribute__((always_inline)) {
        return (unsigned)(lds_off_kmajor(wm0 + l15, ks * 4 + q * 2 + (lg >> 1)) + ((lg & 1) << 3));
    };
    auto frag_b_nt = [&](int ks, int q) __attribute__((always_inline)) {
        return (unsigned)(lds_off_kmajor(wn0 + l15, ks * 4 + q * 2 + (lg >> 1)) + ((lg & 1) << 3));
    };
    auto frag_b_nn = [&](int j) __attribute__((always_inline)) {
        const int k = (lg >> 1) * 8 + (lg & 1) * 4 + (l15 >> 2), n = wn0 + j * 16 + ((l15 & 3) << 2);
        return (unsigned)(lds_off_nmajor16<BN>(k, n >> 3) + ((n & 7) << 1));
    };
    // nks 32-wide k-steps over the register-staged tile; rows: bit i set = this wavefront's 16-row
    // block i may hold non-zero activation rows
    auto compute = [&](int ks0, int nks, unsigned rows) __attribute__((always_inline)) {
        for (int ks = ks0; ks < ks0 + nks; ++ks) {
            const unsigned va0 = lds0 + frag_a(ks, 0), va1 = lds0 + frag_a(ks, 1);
            if constexpr (!NN) {
                const unsigned vb0 = lds0 + TT::UNIT + frag_b_nt(ks, 0), vb1 = lds0 + TT::UNIT + frag_b_nt(ks, 1);
                if constexpr (NBLK == 8)
                    asm volatile(SYMB_GEMM16_KSTEP32_NT : : "v"(va0), "v"(va1), "v"(vb0), "v"(vb1), "s"(rows)
                                 : "memory", "scc", SYMB_GEMM16_VCLOBBERS, SYMB_GEMM16_ACLOBBERS);
                else
                    asm volatile(SYMB_GEMM16S_KSTEP32_NT : : "v"(va0), "v"(va1), "v"(vb0), "v"(vb1), "s"(rows)
                                 : "memory", "scc", SYMB_GEMM16S_VCLOBBERS, SYMB_GEMM16S_ACLOBBERS);
            } else {
                unsigned vb[NBLK];
#pragma unroll
                for (int j = 0; j < NBLK; ++j) vb[j] = lds0 + TT::UNIT + frag_b_nn(j) + ks * 32 * (BN * 2);
                if constexpr (NBLK == 8)
                    asm volatile(SYMB_GEMM16_KSTEP32_NN : : "v"(va0), "v"(va1), "v"(vb[0]), "v"(vb[1]), "v"(vb[2]), "v"(vb[3]),
                                 "v"(vb[4]), "v"(vb[5]), "v"(vb[6]), "v"(vb[7]), "s"(rows)
                                 : "memory", "scc", SYMB_GEMM16_VCLOBBERS, SYMB_GEMM16_ACLOBBERS);
                else
                    asm volatile(SYMB_GEMM16S_KSTEP32_NN : : "v"(va0), "v"(va1), "v"(vb[0]), "v"(vb[1]), "v"(vb[2]), "v"(vb[3]), "s"(rows)
                                 : "memory", "scc", SYMB_GEMM16S_VCLOBBERS, SYMB_GEMM16S_ACLOBBERS);
            }
        }
    };

    // ---- main loop over the full 64-k stages (gemm16_asm.hpp)
    const int KFT = p.K / 64;                              // full stages of the whole K extent
    const int st0 = (int)((long long)KFT * part / nparts);
    const int KF = (int)((long long)KFT * (part + 1) / nparts) - st0;   // this workgroup's stages: [st0, st0 + KF)
    if (KF == 0) {                                         // otherwise the main loop zeroes them
        if constexpr (NBLK == 8) asm volatile(SYMB_GEMM16_ZERO ::: SYMB_GEMM16_ACLOBBERS);
        else asm volatile(SYMB_GEMM16S_ZERO ::: SYMB_GEMM16S_ACLOBBERS);
    }
    if (KF > 0) {
        constexpr int NVB = NBLK > 4 ? NBLK : 4;
        unsigned vA[4], vB[NVB];
#pragma unroll
        for (int j = 0; j < 4; ++j) vA[j] = lds0 + frag_a(j >> 1, j & 1);
#pragma unroll
        for (int j = 0; j < NVB; ++j) vB[j] = lds0 + (NN ? frag_b_nn(j % NBLK) : frag_b_nt((j >> 1) & 1, j & 1));
        // Global byte offsets of this lane's NBLK loads per operand and stage.  One load instruction
        // fills 1 KiB of consecutive LDS: 8 rows of a K-contiguous unit or 1024 / (2 BN) k-rows of the
        // N-contiguous unit; the lane -> chunk map is the inverse of the LDS swizzle.  Rows / columns
        // outside the problem are clamped onto the last valid one and never stored.
        unsigned ab[NBLK], bb[NBLK];
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            const int row = (wave * NBLK + j) * 8 + (lane >> 3), kc = (lane & 7) ^ swz_row(row);
            ab[j] = ((unsigned)(a_row(min(m0 + row, p.M - 1)) - a_tile) + kc * 8) * 2u;
            if constexpr (!NN) {
                bb[j] = ((unsigned)(min(n0 + row, p.N - 1) - n0) * (unsigned)p.K + kc * 8) * 2u;
            } else {
                constexpr int CPR = BN / 8;                     // 16-byte chunks per k-row
                const int krow = (wave * NBLK + j) * (64 / CPR) + lane / CPR, nc = (lane % CPR) ^ swz_nmajor16(krow);
                bb[j] = ((unsigned)krow * (unsigned)p.N + (unsigned)min(nc * 8, p.N - 8 - n0)) * 2u;
            }
        }
        const unsigned long long ga = (unsigned long long)(a_tile + (size_t)st0 * 64);
        const unsigned long long gb = (unsigned long long)(b_tile + (NN ? (size_t)st0 * 64 * p.N : (size_t)st0 * 64));
        const unsigned stride_b = NN ? 128u * (unsigned)p.N : 128u;
        const unsigned swa = (unsigned)__builtin_amdgcn_readfirstlane((int)lds0 + wave * (1024 * NBLK));
        if constexpr (NBLK == 8) {
#define SYMB_GEMM16_LOOP_OPERANDS                                                                                   \
    :                                                                                                              \
    : "v"(vA[0]), "v"(vA[1]), "v"(vA[2]), "v"(vA[3]), "v"(vB[0]), "v"(vB[1]), "v"(vB[2]), "v"(vB[3]), "v"(vB[4]),  \
      "v"(vB[5]), "v"(vB[6]), "v"(vB[7]), "v"(ab[0]), "v"(ab[1]), "v"(ab[2]), "v"(ab[3]), "v"(ab[4]), "v"(ab[5]), "v"(ab[6]), "v"(ab[7]),  \
      "v"(bb[0]), "v"(bb[1]), "v"(bb[2]), "v"(bb[3]), "v"(bb[4]), "v"(bb[5]), "v"(bb[6]), "v"(bb[7]),              \
      "s"(ga), "s"(gb), "s"(stride_b), "s"(KF), "s"(swa)                                                           \
    : "memory", "scc", SYMB_GEMM16_SCLOBBERS, SYMB_GEMM16_VCLOBBERS, SYMB_GEMM16_ACLOBBERS
            if constexpr (NN) asm volatile(SYMB_GEMM16_LOOP_NN SYMB_GEMM16_LOOP_OPERANDS);
            else asm volatile(SYMB_GEMM16_LOOP_NT SYMB_GEMM16_LOOP_OPERANDS);
#undef SYMB_GEMM16_LOOP_OPERANDS
        } else {
#define SYMB_GEMM16S_LOOP_OPERANDS                                                                                  \
    :                                                                                                              \
    : "v"(vA[0]), "v"(vA[1]), "v"(vA[2]), "v"(vA[3]), "v"(vB[0]), "v"(vB[1]), "v"(vB[2]), "v"(vB[3]),              \
      "v"(ab[0]), "v"(ab[1]), "v"(ab[2]), "v"(ab[3]), "v"(bb[0]), "v"(bb[1]), "v"(bb[2]), "v"(bb[3]),              \
      "s"(ga), "s"(gb), "s"(stride_b), "s"(KF), "s"(swa)                                                           \
    : "memory", "scc", SYMB_GEMM16_SCLOBBERS, SYMB_GEMM16S_VCLOBBERS, SYMB_GEMM16S_ACLOBBERS
            if constexpr (NN) asm volatile(SYMB_GEMM16S_LOOP_NN SYMB_GEMM16S_LOOP_OPERANDS);
            else asm volatile(SYMB_GEMM16S_LOOP_NT SYMB_GEMM16S_LOOP_OPERANDS);
#undef SYMB_GEMM16S_LOOP_OPERANDS
        }
        __builtin_amdgcn_s_barrier();                      // everything landed and read before LDS is reused
    }
    if (last_part && KFT * 64 < p.K) {
        gload_tail(KFT * 64);
        lds_store_a();
        lds_store_b();
        __syncthreads();
        compute(0, (p.K - KFT * 64 + 31) >> 5, (1u << NBLK) - 1);
        __syncthreads();
    }

    // ---- output staging: the bf16 tile goes through LDS and leaves as whole 512-byte rows
    const unsigned c_lane = (unsigned)((wm0 + l15) * CP + (wn0 + lg * 4) * 2);   // this lane's C[.][.] of block (0, 0)
    auto stage_out = [&](bf16* __restrict__ dst, bool scale_ia3) __attribute__((always_inline)) {
        if (PLAIN || (!p.bias && !scale_ia3 && !p.neff)) {
            if constexpr (NBLK == 8) asm volatile(SYMB_GEMM16_STAGE_OUT : : "v"(lds0 + c_lane) : "memory", SYMB_GEMM16_VCLOBBERS);
            else asm volatile(SYMB_GEMM16S_STAGE_OUT : : "v"(lds0 + c_lane) : "memory", SYMB_GEMM16S_VCLOBBERS);
        } else if constexpr (!PLAIN) {
            // bias of this lane's column quads, once; IA3 vector and noise effect of each row's own
            // segment per row block
            const int nq0 = n0 + wn0 + lg * 4;
            uint2 bv[NBLK];
#pragma unroll
            for (int j = 0; j < NBLK; ++j) {
                const int n = nq0 + j * 16;
                bv[j] = (p.bias && n < p.N) ? *reinterpret_cast<const uint2*>(p.bias + n) : make_uint2(0u, 0u);
            }
            static_for<0, NBLK>([&](auto I) __attribute__((always_inline)) {
                constexpr int i = decltype(I)::value;
                const int m = m0 + wm0 + i * 16 + l15;
                const bf16* lrow = nullptr;
                const bf16* nrow = nullptr;
                if ((scale_ia3 || p.neff) && m < p.M) {
                    const int s = seg_of_row(p.off, seg_lo, seg_hi, m);
                    if (scale_ia3 && p.seg[s].kind == p.epi_ia3) lrow = p.seg[s].A;
                    if (p.neff) {
                        const NoiseDesc nd = p.neff[s];
                        if (nd.ptr) nrow = nd.ptr + (size_t)(nd.rows == 1 ? 0 : m - p.off[s]) * p.N;
                    }
                }
                uint2 lv[NBLK], nv[NBLK];
#pragma unroll
                for (int j = 0; j < NBLK; ++j) {
                    const int n = nq0 + j * 16;
                    nv[j] = (nrow && n < p.N) ? *reinterpret_cast<const uint2*>(nrow + n) : make_uint2(0u, 0u);
                    lv[j] = (lrow && n < p.N) ? *reinterpret_cast<const uint2*>(lrow + n) : make_uint2(0x3f803f80u, 0x3f803f80u);
                }
                static_for<0, NBLK>([&](auto J) __attribute__((always_inline)) {
                    constexpr int j = decltype(J)::value;
                    float v0, v1, v2, v3;
                    acc16_read4<4 * (NBLK * i + j)>(v0, v1, v2, v3);
                    if (p.bias) {
                        v0 += bf16_bits_to_f32((unsigned short)(bv[j].x & 0xffffu));
                        v1 += bf16_bits_to_f32((unsigned short)(bv[j].x >> 16));
                        v2 += bf16_bits_to_f32((unsigned short)(bv[j].y & 0xffffu));
                        v3 += bf16_bits_to_f32((unsigned short)(bv[j].y >> 16));
                    }
                    if (scale_ia3) {           // rows of other kinds carry ones (exact)
                        v0 *= bf16_bits_to_f32((unsigned short)(lv[j].x & 0xffffu));
                        v1 *= bf16_bits_to_f32((unsigned short)(lv[j].x >> 16));
                        v2 *= bf16_bits_to_f32((unsigned short)(lv[j].y & 0xffffu));
                        v3 *= bf16_bits_to_f32((unsigned short)(lv[j].y >> 16));
                    }
                    if (p.neff) {              // y = y_noisy - n_eff, still in fp32
                        v0 -= bf16_bits_to_f32((unsigned short)(nv[j].x & 0xffffu));
                        v1 -= bf16_bits_to_f32((unsigned short)(nv[j].x >> 16));
                        v2 -= bf16_bits_to_f32((unsigned short)(nv[j].y & 0xffffu));
                        v3 -= bf16_bits_to_f32((unsigned short)(nv[j].y >> 16));
                    }
                    uint2 o;
                    o.x = pack2_bf16(v0, v1);
                    o.y = pack2_bf16(v2, v3);
                    *reinterpret_cast<uint2*>(smem + c_lane + i * 16 * CP + j * 32) = o;
                });
            });
        }
        __syncthreads();
        const bool to_seg = p.c_seg != nullptr && dst == p.C;   // the final output goes to the segments' own buffers
        constexpr int LPR = BN / 8;                  // lanes per row (16 bytes each)
        constexpr int RPP = 256 / LPR;               // rows per pass of the workgroup
        constexpr int NPASS = BM / RPP, BATCH = NPASS < 16 ? NPASS : 16;
        const int col = (lane % LPR) * 8, r0 = wave * (64 / LPR) + lane / LPR;
        const bool nok = n0 + col < p.N;
        if (!to_seg) {
            // NPASS rows per lane, in batches: up to sixteen LDS reads in flight, then their stores
            bf16* const out0 = dst + (size_t)(m0 + r0) * p.N + n0 + col;
#pragma unroll
            for (int part = 0; part < NPASS / BATCH; ++part) {
                uint4 v[BATCH];
#pragma unroll
                for (int q = 0; q < BATCH; ++q) v[q] = *reinterpret_cast<const uint4*>(smem + (r0 + (part * BATCH + q) * RPP) * CP + col * 2);
#pragma unroll
                for (int q = 0; q < BATCH; ++q) {
                    const int r = r0 + (part * BATCH + q) * RPP;
                    if (nok && m0 + r < p.M) *reinterpret_cast<uint4*>(out0 + (size_t)((part * BATCH + q) * RPP) * p.N) = v[q];
                }
            }
        } else {
#pragma unroll 4
            for (int r = r0; r < BM; r += RPP) {
                const int m = m0 + r;
                if (m < p.M && nok) {
                    const int s = seg_of_row(p.off, seg_lo, seg_hi, m);
                    bf16* rowp = p.c_seg[s] + (size_t)(m - p.off[s]) * p.N;
                    *reinterpret_cast<uint4*>(rowp + n0 + col) = *reinterpret_cast<const uint4*>(smem + r * CP + col * 2);
                }
            }
        }
    };

    // ---- optional store of the pre-adapter output (accumulator + bias, before the LoRA term)
    if constexpr (!PLAIN) {
        if (p.Cbase) {
            stage_out(p.Cbase, false);
            __syncthreads();                         // LDS is reused by the LoRA tiles below
        }
    }

    // ---- LoRA term: extra 32-wide k-steps per LoRA segment that meets this row tile.  Several steps
    // are in flight, each in a register set of its own: the loads of the first went out before the main
    // loop, those of the others go out here, and each step, once its registers are in LDS, requests the
    // next step that has no registers yet into them.  (A step computes little; with one step in flight
    // every step waited out its own loads.)  One barrier per
    // step is enough because consecutive steps use different halves of the staged tile: whoever stores
    // step k + 1 has passed the barrier of step k, which every wavefront reaches after its MFMAs of
    // step k - 1, the last reader of that half.
    // (ESETS steps are in flight: two on a K-contiguous weight and one on an N-contiguous one for the
    // 256x256 tile, which has no registers left for more; one more each for the 128x128 tile.  Step k
    // uses set k % ESETS and half k % 2.)
    if (e_have[0]) {
        static_for<1, ESETS>([&](auto J) __attribute__((always_inline)) {
            constexpr int j = decltype(J)::value;
            e_have[j] = ext_more;
            if (e_have[j]) ext_load(J);
        });
        auto ext_step = [&](auto SETC, auto HALFC, bool& have) __attribute__((always_inline)) {
            constexpr int SET = decltype(SETC)::value, HALF = decltype(HALFC)::value;
            // this wavefront's 16-row blocks that hold rows of the step's segment (the other rows of the
            // activation-side tile are zero)
            constexpr unsigned ALL = (1u << NBLK) - 1;
            const int r_lo = e_rlo[SET], r_hi = e_rhi[SET];
            const int b_lo = max(r_lo - (m0 + wm0), 0) >> 4, b_hi = min((r_hi - 1 - (m0 + wm0)) >> 4, NBLK - 1);
            const unsigned rows = (unsigned)__builtin_amdgcn_readfirstlane(
                (r_hi > m0 + wm0 && b_lo <= b_hi) ? (int)((ALL >> (NBLK - 1 - b_hi)) & (ALL << b_lo) & ALL) : 0);
#pragma unroll
            for (int i = 0; i < EC; ++i) {
                *reinterpret_cast<uint4*>(sA + e_lds[HALF] + i * 8192) = ea[SET][i];
                if constexpr (!NN) *reinterpret_cast<uint4*>(sB + e_lds[HALF] + i * 8192) = eb[SET][i];
                else *reinterpret_cast<uint4*>(sB + b_lds0 + (HALF * 32 + i * KSTEP) * (BN * 2)) = eb[SET][i];
            }
            __syncthreads();
            have = ext_more;
            if (have) ext_load(SETC);
            compute(HALF, 1, rows);
        };
        // steps run in the order they were requested, so the first empty set ends the loop
        constexpr int EPERIOD = (ESETS & 1) ? 2 * ESETS : ESETS;
        bool ext_done = false;
        while (!ext_done) {
            static_for<0, EPERIOD>([&](auto K) __attribute__((always_inline)) {
                constexpr int k = decltype(K)::value;
                if (ext_done) return;
                if (!e_have[k % ESETS]) { ext_done = true; return; }
                ext_step(std::integral_constant<int, k % ESETS>{}, std::integral_constant<int, k & 1>{}, e_have[k % ESETS]);
            });
        }
        __syncthreads();                             // LDS goes to the output tile / the arrival flag next
    }

    // ---- K-split tile: every part leaves its accumulators in the workspace (register order: 1 KiB
    // per wavefront and 16x16 block); the part that arrives last adds all of them up in part order
    // (so the sum does not depend on who was last) and writes the tile.
    if (nparts > 1) {
        constexpr int PT = BM * BN;                  // floats per partial tile
        float* const tile_parts = p.partial + (size_t)slot * nparts * PT;
        const unsigned lane_off = (unsigned)(wave * (NBLK * NBLK * 1024) + lane * 16);
        const unsigned long long mine = (unsigned long long)(tile_parts + (size_t)part * PT);
        if constexpr (NBLK == 8) asm volatile(SYMB_GEMM16_STORE_PARTIAL : : "v"(lane_off), "s"(mine) : "memory", SYMB_GEMM16_VCLOBBERS);
        else asm volatile(SYMB_GEMM16S_STORE_PARTIAL : : "v"(lane_off), "s"(mine) : "memory", SYMB_GEMM16S_VCLOBBERS);
        // No device-scope fence (on this chip it writes back and invalidates the XCD's whole L2, tens
        // of microseconds with the outputs of other tiles in it).  None is needed: the parts of a tile
        // run on one XCD (same blockIdx & 7), i.e. behind one L2; the template above returns when its
        // stores are acknowledged by that L2 (write-through L1); the counter is bumped after that;
        // and the reader's L1 holds no line of the partial tiles (nobody read them in this launch).
        __syncthreads();
        int* const flag = reinterpret_cast<int*>(smem);
        if (tid == 0) {
            const int seen = atomicAdd(p.k_count + slot, 1);
            // the last arrival leaves the counter as it found the launch: zero, for the next one
            if (seen == nparts - 1) __hip_atomic_store(p.k_count + slot, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = seen;
        }
        __syncthreads();
        const bool last_arrival = *flag == nparts - 1;
        __syncthreads();                             // the flag's LDS word is part of the staging tile
        if (!last_arrival) return;
        const float4* src = reinterpret_cast<const float4*>(tile_parts) + wave * (NBLK * NBLK * 64) + lane;
        // Blocks are requested in groups (the accumulator writes below are assembly statements, which the
        // loads could not be moved across): sixteen blocks of one part at a time, or, with at most four
        // parts, eight blocks of all parts at once, which halves the number of round trips.
        if (nparts <= 4) {
            static_for<2, 5>([&](auto NPC) __attribute__((always_inline)) {
                constexpr int NP = decltype(NPC)::value;
                if (nparts != NP) return;
                static_for<0, NBLK * NBLK / 8>([&](auto G) __attribute__((always_inline)) {
                    constexpr int g = decltype(G)::value;
                    float4 v[NP][8];
#pragma unroll
                    for (int q = 0; q < NP; ++q)
#pragma unroll
                        for (int b = 0; b < 8; ++b) v[q][b] = src[(size_t)q * (PT / 4) + (g * 8 + b) * 64];
#pragma unroll
                    for (int q = 1; q < NP; ++q)
#pragma unroll
                        for (int b = 0; b < 8; ++b) { v[0][b].x += v[q][b].x; v[0][b].y += v[q][b].y; v[0][b].z += v[q][b].z; v[0][b].w += v[q][b].w; }
                    static_for<0, 8>([&](auto B) __attribute__((always_inline)) {
                        constexpr int b = decltype(B)::value;
                        acc16_write4<4 * (g * 8 + b)>(v[0][b].x, v[0][b].y, v[0][b].z, v[0][b].w);
                    });
                });
            });
        } else {
            static_for<0, NBLK * NBLK / 16>([&](auto G) __attribute__((always_inline)) {
                constexpr int g = decltype(G)::value;
                float4 sum[16];
#pragma unroll
                for (int b = 0; b < 16; ++b) sum[b] = src[(g * 16 + b) * 64];
                for (int q = 1; q < nparts; ++q) {
                    float4 v[16];
#pragma unroll
                    for (int b = 0; b < 16; ++b) v[b] = src[(size_t)q * (PT / 4) + (g * 16 + b) * 64];
#pragma unroll
                    for (int b = 0; b < 16; ++b) { sum[b].x += v[b].x; sum[b].y += v[b].y; sum[b].z += v[b].z; sum[b].w += v[b].w; }
                }
                static_for<0, 16>([&](auto B) __attribute__((always_inline)) {
                    constexpr int b = decltype(B)::value;
                    acc16_write4<4 * (g * 16 + b)>(sum[b].x, sum[b].y, sum[b].z, sum[b].w);
                });
            });
        }
    }

    // ---- final output: bias, IA3 scale, noise effect, one rounding, whole-row stores
    stage_out(p.C, p.epi_ia3 != 0 && p.tile_epi[tm] != 0);
}

}  // namespace symb
