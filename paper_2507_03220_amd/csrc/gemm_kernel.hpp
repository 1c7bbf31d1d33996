// bf16 MFMA GEMM of the frozen base weight with the per-segment adapter fused in.
//
//   forward  (NN = false):  C[m][n] = sum_k Aop[m][k] * Bop[n][k]   (Bop = W [d_out][d_in], K-contiguous)
//   backward (NN = true) :  C[m][n] = sum_k Aop[m][k] * Bop[k][n]   (Bop = W [d_out][d_in], N-contiguous)
//
// plus, for every LoRA segment that meets the row tile, extra K-steps
//   forward : C += Hs[m][p] * B_i[n][p]      (Hs = s_i * X A_i^T from the shrink kernel)
//   backward: C += dH[m][p] * A_i[p][n]      (dH = s_i * dY B_i)
// where Hs / dH arrive as a bf16 value plus a bf16 rounding residual (two K-steps per rank block),
// accumulated in the same fp32 accumulators before the single rounding to bf16, and an
// epilogue with the optional bias, the optional store of the pre-adapter output and
// the IA3 per-channel scale of each row's own segment.
//
// Two kernels compute this.  Large problems: symb_gemm16_kernel (gemm16_kernel.hpp), a 256x256 tile
// with a hand-scheduled assembly main loop.  Small problems: symb_gemm_kernel below, instantiated
// for a 128x128 tile.  Tiling of the kernel below (gfx950): one workgroup owns a BM x BN tile of C;
// WGM x WGN wavefronts of 64 lanes each own a (BM/WGM) x (BN/WGN) sub-tile as 32x32 blocks of
// v_mfma_f32_32x32x16_bf16.  Operands go from global memory straight into an LDS ring (no register
// hop) in 32-k stages, with a compiler-scheduled loop.  The MFMA is issued as (weight fragment,
// activation fragment), so a lane ends up holding, for one row m, runs of 4 consecutive n: rows
// keep their own segment in the epilogue, which stages the bf16 tile through LDS and writes whole
// rows.  This file also holds what both kernels share: the parameter block, the LDS layout of a
// K-contiguous 64-k tile and the predicated 16-byte load.
#pragma once
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
                                // (IA3 in the forward, IA3_IN in the input gradient)
    // Per-segment buffers instead of flat tensors (device arrays of S pointers, or null): row t of
    // segment i is a_seg[i] + (t - off[i]) * K resp. c_seg[i] + (t - off[i]) * N.  All a_seg buffers lie
    // within 4 GiB above a_base (checked by the host), so lane offsets from a_base fit 32 bits.
    const bf16* const* a_seg;
    const bf16* a_base;
    bf16* const* c_seg;
    const NoiseDesc* neff;      // device [S] or null: per-segment noise effect subtracted last (privacy flow)
    // K-split (symb_gemm16_kernel only; k_parts <= 1: off): every tile is computed by k_parts
    // workgroups; partial holds k_parts fp32 tiles per tile, k_count one zeroed arrival counter per tile.
    int k_parts;
    float* partial;
    int* k_count;
    int walk;                   // 0: each XCD walks one contiguous run of tiles; 1: rounds of 32 tiles dealt to the XCDs in turn
    double timing_flops;        // host bookkeeping for the measurement hook; unused on the device
#ifdef SYMB_GEMM_TRACE
    unsigned long long* trace;  // tuning builds only: 16 timestamp slots per tile
#endif
#ifdef SYMB_GEMM_PROBE
    int probe;                  // tuning builds only (256x256 kernel): 1 = no in-loop global loads, 2 = nor LDS reads, 5 = nor barriers
#endif
};

constexpr int GEMM_BK = 64;       // k per register-staged tile (K remainder, LoRA term)
constexpr int GEMM_SK = 32;       // k per main-loop stage (direct global -> LDS)
constexpr int GEMM_NSTAGE = 4;    // main-loop LDS ring depth

// s_waitcnt immediates (gfx9 encoding: vmcnt [3:0]+[15:14], expcnt [6:4], lgkmcnt [11:8]).
__device__ __host__ constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }
__device__ __host__ constexpr int lgkmcnt0_mask() { return ~0x0F00; }

// 16-byte chunk swizzle of a K-contiguous tile row (8 chunks of 8 bf16 per row).
__device__ __forceinline__ int swz_row(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int BM, int BN, int WGM, int WGN, bool NN>
struct GemmTile {
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int BK = GEMM_BK;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int A_STAGE = BM * GEMM_SK * 2, B_STAGE = BN * GEMM_SK * 2, STAGE_BYTES = A_STAGE + B_STAGE;
    static constexpr int C_PITCH = BN * 2 + 16, C_BYTES = BM * C_PITCH;     // epilogue staging of the bf16 tile
    static constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;   // 16-byte chunks per thread per K-step
    static constexpr int SK = GEMM_SK;                         // k per main-loop stage
    static constexpr int SMEM_RING = GEMM_NSTAGE * STAGE_BYTES;
    static constexpr int SMEM_IN = (2 * (A_BYTES + B_BYTES) > SMEM_RING) ? 2 * (A_BYTES + B_BYTES) : SMEM_RING;
    static constexpr int SMEM = SMEM_IN > C_BYTES ? SMEM_IN : C_BYTES;
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tile must be made of 32x32 blocks");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "tile chunks must divide over the threads");
};

// ---- LDS addressing --------------------------------------------------------------------------
// K-contiguous tile: [rows][64] bf16, 128 B per row, chunk kc stored at kc ^ swz_row(row).
__device__ __forceinline__ int lds_off_kmajor(int row, int kc) { return row * 128 + ((kc ^ swz_row(row)) << 4); }
// N-contiguous tile (NN weight): [64 k][BN] bf16, chunk nc of row k stored at nc ^ ((k & 3) << 2).
template <int BN>
__device__ __forceinline__ int lds_off_nmajor(int k, int nc) { return k * (BN * 2) + ((nc ^ ((k & 3) << 2)) << 4); }

__device__ __forceinline__ bf16x8 lds_read_frag_kmajor(const unsigned char* buf, int row, int kc) {
    return *reinterpret_cast<const bf16x8*>(buf + lds_off_kmajor(row, kc));
}
// K-contiguous main-loop stage: [rows][32] bf16, 64 B per row, chunk kc (0..3) stored at kc ^ ((row >> 2) & 3):
// 16 consecutive rows at one kc then hit 16 different 16-byte bank groups.
__device__ __forceinline__ bf16x8 lds_read_frag_k32(const unsigned char* buf, int row, int kc) {
    return *reinterpret_cast<const bf16x8*>(buf + row * 64 + ((kc ^ ((row >> 2) & 3)) << 4));
}

// Fragment of a 32(n) x 16(k) block out of an N-contiguous tile via the transposing LDS read:
// lane l ends with n = nb + (l & 31), k = k16 + 8*(l >> 5) + 0..7.
template <int BN>
__device__ __forceinline__ bf16x8 lds_read_frag_nmajor(const unsigned char* buf, int nb, int k16, int lane) {
    const int g = lane >> 4, jj = lane & 15;
    const int n = nb + ((g & 1) << 4) + ((jj & 3) << 2);
    const int k = k16 + ((g >> 1) << 3) + (jj >> 2);
    const unsigned char* p0 = buf + lds_off_nmajor<BN>(k, n >> 3) + ((n & 7) << 1);
    const unsigned char* p1 = buf + lds_off_nmajor<BN>(k + 4, n >> 3) + ((n & 7) << 1);
    typedef __attribute__((address_space(3))) shortx4 lds_s4;
    shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p0));
    shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p1));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short shortx8;
    shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// The same fragment, requested without the compiler knowing it is an LDS read: lo / hi are valid only
// after a later s_waitcnt lgkmcnt(0).  For the main loop, whose stages arrive by LDS DMA
// (global_load_lds): there the compiler makes every transposing LDS read (an intrinsic without
// memory operands) wait for all DMA loads in flight, the next stages' included, which serialises
// the loop on memory latency.  The loop's own waits and barriers already order these reads after
// the DMA of their stage.
template <int BN>
__device__ __forceinline__ void lds_request_frag_nmajor(const unsigned char* buf, int nb, int k16, int lane, uint2& lo, uint2& hi) {
    const int g = lane >> 4, jj = lane & 15;
    const int n = nb + ((g & 1) << 4) + ((jj & 3) << 2);
    const int k = k16 + ((g >> 1) << 3) + (jj >> 2);
    const unsigned a = (unsigned)(size_t)(buf + lds_off_nmajor<BN>(k, n >> 3) + ((n & 7) << 1));
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(a));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a), "n"(4 * BN * 2));   // 4 k-rows down: same swizzle
}

__device__ __forceinline__ uint4 ld_global_16(const bf16* p, bool ok) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (ok) v = *reinterpret_cast<const uint4*>(p);
    return v;
}

template <int BM, int BN, int WGM, int WGN, bool NN>
__global__ void __launch_bounds__(WGM * WGN * 64)
symb_gemm_kernel(const GemmParams p) {
    using TT = GemmTile<BM, BN, WGM, WGN, NN>;
    constexpr int NT = TT::NT, BK = TT::BK, MB = TT::MB, NB = TT::NB, CA = TT::CA, CB = TT::CB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* const sA = smem;                       // two A buffers
    unsigned char* const sB = smem + 2 * TT::A_BYTES;     // two B buffers

    // ---- tile of this workgroup: consecutive workgroup ids go to different XCDs, so give every
    // XCD one contiguous run of tiles, walked in groups of group_m row tiles per column tile.
    const int total = p.num_m_tiles * p.num_n_tiles;
    int lin;
    if (p.walk == 1) {
        // rounds of 32 tiles (one per CU of an XCD) dealt to the XCDs in turn: the eight XCDs work
        // on neighbouring 8x4 blocks of the same row-tile group at the same time
        const int k = blockIdx.x >> 3;
        lin = (((k >> 5) << 3) + (blockIdx.x & 7)) * 32 + (k & 31);
        if (lin >= total) return;
    } else {
        const int per_xcd = (total + 7) >> 3;
        lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
        if (lin >= total || (int)(blockIdx.x >> 3) >= per_xcd) return;
    }
    const int width = p.group_m * p.num_n_tiles;
    const int first_m = (lin / width) * p.group_m;
    const int gsz = min(p.num_m_tiles - first_m, p.group_m);
    const int tm = first_m + (lin % width) % gsz;
    const int tn = (lin % width) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;

#ifdef SYMB_GEMM_TRACE
    if (p.trace && threadIdx.x == 0) { p.trace[(size_t)lin * 16 + 0] = __builtin_amdgcn_s_memrealtime(); p.trace[(size_t)lin * 16 + 5] = __builtin_readcyclecounter(); }
#endif
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * TT::WTM, wn0 = (wave % WGN) * TT::WTN;
    // segment range of this row tile, fetched now so that its latency hides under the main loop
    const int seg_lo = p.tile_seg_lo[tm], seg_hi = p.tile_seg_hi[tm];
    // row m (< M) of the activation operand: in the flat tensor or in its segment's own buffer
    auto a_row = [&](int m) __attribute__((always_inline)) -> const bf16* {
        if (!p.a_seg) return p.Aop + (size_t)m * p.K;
        const int s = seg_of_row(p.off, seg_lo, seg_hi, m);
        return p.a_seg[s] + (size_t)(m - p.off[s]) * p.K;
    };
    // loads address their rows as 32-bit offsets from this pointer
    const bf16* const a_tile = p.a_seg ? p.a_base : p.Aop + (size_t)m0 * p.K;

    floatx16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- per-thread staging slots.  Chunk i of a thread sits NT/8 rows (K-contiguous tiles) or
    // NT/(BN/8) k-rows (N-contiguous weight tile) below chunk 0, in the same 16-byte column, so one
    // LDS offset per operand is enough (the swizzles repeat every 16 rows / 4 k-rows).
    constexpr int RSTEP = NT / 8;                 // row step between a thread's chunks, K-contiguous tile
    constexpr int KSTEP = NT / (BN / 8);          // k-row step, N-contiguous tile
    static_assert(RSTEP % 16 == 0 && (!NN || KSTEP % 4 == 0), "chunk stride must preserve the LDS swizzle");
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;
    const int nn_k = tid / (BN / 8), nn_nc = tid % (BN / 8);
    const int a_lds0 = lds_off_kmajor(lrow, tid & 7);
    const int b_lds0 = NN ? lds_off_nmajor<BN>(nn_k, nn_nc) : a_lds0;

    uint4 ra[CA], rb[CB];
    auto lds_store_a = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < CA; ++i) *reinterpret_cast<uint4*>(sA + buf * TT::A_BYTES + a_lds0 + i * RSTEP * 128) = ra[i];
    };
    auto lds_store_b = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            if constexpr (!NN) *reinterpret_cast<uint4*>(sB + buf * TT::B_BYTES + b_lds0 + i * RSTEP * 128) = rb[i];
            else *reinterpret_cast<uint4*>(sB + buf * TT::B_BYTES + b_lds0 + i * KSTEP * (BN * 2)) = rb[i];
        }
    };
    auto lds_store = [&](int buf) __attribute__((always_inline)) {
        lds_store_a(buf);
        lds_store_b(buf);
    };

    // ---- main-loop staging: global memory -> LDS directly (no registers), NSTAGE stages of SK = 32
    // k each.  One such load instruction moves 16 bytes per lane into 1 KiB of consecutive LDS, so
    // the lane -> global chunk map below is the inverse of the LDS swizzle.  No predicates: a row
    // (column chunk) outside the problem is clamped onto the last valid one and never stored.
    // Offsets are 32-bit element offsets from a wave-uniform tile pointer that advances per stage.
    constexpr int NW = NT / 64;
    constexpr int AI = BM / 16 / NW, BI = BN / 16 / NW;       // load instructions per wave per stage
    static_assert(AI >= 1 && BI >= 1, "tile too small for this many wavefronts");
    unsigned a_off[AI], b_off[BI];
#pragma unroll
    for (int j = 0; j < AI; ++j) {
        const int row = (wave * AI + j) * 16 + (lane >> 2), kc = (lane & 3) ^ ((row >> 2) & 3);
        a_off[j] = (unsigned)(a_row(min(m0 + row, p.M - 1)) - a_tile) + kc * 8;
    }
#pragma unroll
    for (int j = 0; j < BI; ++j) {
        if constexpr (!NN) {
            const int row = (wave * BI + j) * 16 + (lane >> 2), kc = (lane & 3) ^ ((row >> 2) & 3);
            b_off[j] = (unsigned)(min(n0 + row, p.N - 1) - n0) * (unsigned)p.K + kc * 8;
        } else {
            constexpr int CPR = BN / 8;                        // 16-byte chunks per k-row
            const int krow = (wave * BI + j) * (64 / CPR) + lane / CPR, nc = (lane % CPR) ^ ((krow & 3) << 2);
            b_off[j] = (unsigned)krow * (unsigned)p.N + (unsigned)min(nc * 8, p.N - 8 - n0);
        }
    }
    const bf16* const b_tile = NN ? (p.Bop + n0) : (p.Bop + (size_t)n0 * p.K);
    typedef __attribute__((address_space(3))) void lds_void_t;
    typedef __attribute__((address_space(1))) const void glb_void_t;
    auto stage_issue = [&](int stage, int ks32) __attribute__((always_inline)) {
        unsigned char* sa = smem + stage * TT::STAGE_BYTES;
        unsigned char* sb = sa + TT::A_STAGE;
        const bf16* at = a_tile + (size_t)ks32 * GEMM_SK;
        const bf16* bt = NN ? (b_tile + (size_t)ks32 * GEMM_SK * p.N) : (b_tile + (size_t)ks32 * GEMM_SK);
#pragma unroll
        for (int j = 0; j < AI; ++j)
            __builtin_amdgcn_global_load_lds((glb_void_t*)(at + a_off[j]), (lds_void_t*)(sa + (wave * AI + j) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < BI; ++j)
            __builtin_amdgcn_global_load_lds((glb_void_t*)(bt + b_off[j]), (lds_void_t*)(sb + (wave * BI + j) * 1024), 16, 0, 0);
    };
    // Predicated, zero-filling variant for the K remainder (K % 64 != 0).
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

    // MFMA fragments, double buffered in registers across the 16-wide k-steps.
    bf16x8 xa[2][MB], wb[2][NB];
    // from a 64-k tile staged through registers (K remainder, LoRA term)
    auto load_frags = [&](int buf, int ks, int set) __attribute__((always_inline)) {
        const unsigned char* bufA = sA + buf * TT::A_BYTES;
        const unsigned char* bufB = sB + buf * TT::B_BYTES;
#pragma unroll
        for (int i = 0; i < MB; ++i)
            xa[set][i] = lds_read_frag_kmajor(bufA, wm0 + i * 32 + (lane & 31), ks * 2 + (lane >> 5));
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if constexpr (!NN) wb[set][j] = lds_read_frag_kmajor(bufB, wn0 + j * 32 + (lane & 31), ks * 2 + (lane >> 5));
            else wb[set][j] = lds_read_frag_nmajor<BN>(bufB, wn0 + j * 32, ks * 16, lane);
        }
    };
    // from a 32-k main-loop stage.  N-contiguous weight: the fragments are only requested here
    // (halves in wlo / whi); settle(set) waits for them and puts them together.
    uint2 wlo[2][NB], whi[2][NB];
    auto load_frags32 = [&](int stage, int ks, int set) __attribute__((always_inline)) {
        const unsigned char* bufA = smem + stage * TT::STAGE_BYTES;
        const unsigned char* bufB = bufA + TT::A_STAGE;
#pragma unroll
        for (int i = 0; i < MB; ++i)
            xa[set][i] = lds_read_frag_k32(bufA, wm0 + i * 32 + (lane & 31), ks * 2 + (lane >> 5));
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if constexpr (!NN) wb[set][j] = lds_read_frag_k32(bufB, wn0 + j * 32 + (lane & 31), ks * 2 + (lane >> 5));
            else lds_request_frag_nmajor<BN>(bufB, wn0 + j * 32, ks * 16, lane, wlo[set][j], whi[set][j]);
        }
    };
    auto settle = [&](int set) __attribute__((always_inline)) {
        if constexpr (NN) {
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(wlo[set][0]), "+v"(whi[set][0]));
#pragma unroll
            for (int j = 1; j < NB; ++j) asm volatile("" : "+v"(wlo[set][j]), "+v"(whi[set][j]));   // valid from here on as well
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const uint4 v = make_uint4(wlo[set][j].x, wlo[set][j].y, whi[set][j].x, whi[set][j].y);
                wb[set][j] = __builtin_bit_cast(bf16x8, v);
            }
        }
    };
    auto mfma_set = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[set][j], xa[set][i], acc[i][j], 0, 0, 0);
    };
    // Asks the scheduler to issue one LDS fragment read after each MFMA instead of sinking the
    // reads to just before their first use (which would leave the matrix pipe idle for the
    // whole LDS latency once per k-step).
    auto interleave_hint = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < MB + NB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, NN ? 2 : 1, 0);   // then LDS reads
        }
        __builtin_amdgcn_sched_group_barrier(0x008, MB * NB - (MB + NB), 0);
    };
    // Plain (not pipelined) pass over the register-staged tile in buffer 0; K remainder and LoRA term.
    auto compute = [&](int nks) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks < nks) {
                load_frags(0, ks, 0);
                mfma_set(0);
            }
        }
    };

    // ---- main loop over the full stages.  NSTAGE LDS buffers form a ring; the loads of
    // stage t + NSTAGE are issued as soon as every wavefront is done with stage t, i.e. NSTAGE - 1
    // iterations before they are needed.  Per iteration: MFMAs of k-step 0 run while the fragments
    // of k-step 1 are read; then this wavefront's loads of the next stage are awaited, one barrier
    // makes that stage complete for everybody (and frees this one), the refill of this buffer is
    // issued, and the MFMAs of k-step 1 run while the next stage's first fragments are read.
    // Every iteration issues the same number of loads (past the end they refetch the last stage
    // into a buffer nobody reads again), so the vmcnt immediates below stay exact.
    constexpr int NS = GEMM_NSTAGE, LPS = AI + BI;             // loads per wavefront per stage
    constexpr int VM_STEADY = LPS * (NS - 2);                  // younger stages that may stay in flight
    static_assert(LPS * (NS - 1) < 64, "vmcnt is a 6-bit counter");
    const int KF = p.K / TT::SK;                               // full stages
    if (KF > 0) {
#pragma unroll
        for (int t = 0; t < NS; ++t) stage_issue(t, min(t, KF - 1));
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPS * (NS - 1)));
        __builtin_amdgcn_s_barrier();
        load_frags32(0, 0, 0);
#ifdef SYMB_GEMM_TRACE
        if (p.trace && threadIdx.x == 0) p.trace[(size_t)lin * 16 + 1] = __builtin_amdgcn_s_memrealtime();
#endif
        int stage = 0;
        for (int kt = 0; kt < KF; ++kt) {
            const int nxt = (stage + 1 == NS) ? 0 : stage + 1;
            settle(0);
            load_frags32(stage, 1, 1);
            mfma_set(0);
            interleave_hint();
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(VM_STEADY) & lgkmcnt0_mask());
            __builtin_amdgcn_s_barrier();
            stage_issue(stage, min(kt + NS, KF - 1));
            settle(1);
            load_frags32(nxt, 0, 0);
            mfma_set(1);
            interleave_hint();
            stage = nxt;
        }
        settle(0);                                             // the last iteration's request for a stage nobody multiplies
        __builtin_amdgcn_s_waitcnt(0);                         // everything landed before LDS is reused
        __builtin_amdgcn_s_barrier();
#ifdef SYMB_GEMM_TRACE
        if (p.trace && threadIdx.x == 0) p.trace[(size_t)lin * 16 + 2] = __builtin_amdgcn_s_memrealtime();
#endif
    }
    if (KF * TT::SK < p.K) {
        gload_tail(KF * TT::SK);
        lds_store(0);
        __syncthreads();
        compute((p.K - KF * TT::SK + 15) >> 4);
        __syncthreads();
    }

    // ---- output staging.  A lane owns 4 consecutive columns of 32 different rows; stored directly
    // that is 32 partial lines per instruction, so the bf16 tile goes through LDS and leaves as
    // whole 512-byte rows.  The accumulators are only read here: bias and the IA3 scale of each
    // row's own segment are applied on the way out, then one rounding to bf16.
    auto for_each_quad = [&](auto&& fn) __attribute__((always_inline)) {
        // fn(i, j, rg, m, n): this lane holds acc[i][j][rg*4 .. rg*4+3] = C[m][n .. n+3]
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            const int m = m0 + wm0 + i * 32 + (lane & 31);
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int n = n0 + wn0 + j * 32 + rg * 8 + ((lane >> 5) << 2);
                    fn(i, j, rg, m, n);
                }
        }
    };
    constexpr int CP = TT::C_PITCH;                  // bytes per staged row (BN * 2 + 16: bank spread)
    auto read_quad = [&](int i, int j, int rg, float& v0, float& v1, float& v2, float& v3) __attribute__((always_inline)) {
        v0 = acc[i][j][rg * 4 + 0]; v1 = acc[i][j][rg * 4 + 1];
        v2 = acc[i][j][rg * 4 + 2]; v3 = acc[i][j][rg * 4 + 3];
    };
    auto stage_out = [&](bf16* __restrict__ dst, bool scale_ia3) __attribute__((always_inline)) {
        if (!p.bias && !scale_ia3 && !p.neff) {
            for_each_quad([&](int i, int j, int rg, int m, int n) __attribute__((always_inline)) {
                float v0, v1, v2, v3;
                read_quad(i, j, rg, v0, v1, v2, v3);
                uint2 o;
                o.x = pack2_bf16(v0, v1);
                o.y = pack2_bf16(v2, v3);
                *reinterpret_cast<uint2*>(smem + (m - m0) * CP + (n - n0) * 2) = o;
            });
        } else {
            // bias of this lane's 16 column quads, once; IA3 vector of each row's own segment per row block
            const int nq0 = n0 + wn0 + ((lane >> 5) << 2);
            uint2 bv[NB][4];
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int n = nq0 + j * 32 + rg * 8;
                    bv[j][rg] = (p.bias && n < p.N) ? *reinterpret_cast<const uint2*>(p.bias + n) : make_uint2(0u, 0u);
                }
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const int m = m0 + wm0 + i * 32 + (lane & 31);
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
                uint2 lv[NB][4], nv[NB][4];
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int n = nq0 + j * 32 + rg * 8;
                        nv[j][rg] = (nrow && n < p.N) ? *reinterpret_cast<const uint2*>(nrow + n) : make_uint2(0u, 0u);
                    }
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int n = nq0 + j * 32 + rg * 8;
                        lv[j][rg] = (lrow && n < p.N) ? *reinterpret_cast<const uint2*>(lrow + n) : make_uint2(0x3f803f80u, 0x3f803f80u);
                    }
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int n = nq0 + j * 32 + rg * 8;
                        float v0, v1, v2, v3;
                        read_quad(i, j, rg, v0, v1, v2, v3);
                        if (p.bias) {
                            v0 += bf16_bits_to_f32((unsigned short)(bv[j][rg].x & 0xffffu));
                            v1 += bf16_bits_to_f32((unsigned short)(bv[j][rg].x >> 16));
                            v2 += bf16_bits_to_f32((unsigned short)(bv[j][rg].y & 0xffffu));
                            v3 += bf16_bits_to_f32((unsigned short)(bv[j][rg].y >> 16));
                        }
                        if (scale_ia3) {           // rows of other kinds carry ones (exact)
                            v0 *= bf16_bits_to_f32((unsigned short)(lv[j][rg].x & 0xffffu));
                            v1 *= bf16_bits_to_f32((unsigned short)(lv[j][rg].x >> 16));
                            v2 *= bf16_bits_to_f32((unsigned short)(lv[j][rg].y & 0xffffu));
                            v3 *= bf16_bits_to_f32((unsigned short)(lv[j][rg].y >> 16));
                        }
                        if (p.neff) {              // y = y_noisy - n_eff, still in fp32
                            v0 -= bf16_bits_to_f32((unsigned short)(nv[j][rg].x & 0xffffu));
                            v1 -= bf16_bits_to_f32((unsigned short)(nv[j][rg].x >> 16));
                            v2 -= bf16_bits_to_f32((unsigned short)(nv[j][rg].y & 0xffffu));
                            v3 -= bf16_bits_to_f32((unsigned short)(nv[j][rg].y >> 16));
                        }
                        uint2 o;
                        o.x = pack2_bf16(v0, v1);
                        o.y = pack2_bf16(v2, v3);
                        *reinterpret_cast<uint2*>(smem + (m - m0) * CP + (n - n0) * 2) = o;
                    }
            }
        }
#ifdef SYMB_GEMM_TRACE
        if (p.trace && threadIdx.x == 0) p.trace[(size_t)lin * 16 + 8] = __builtin_amdgcn_s_memrealtime();
#endif
        __syncthreads();
#ifdef SYMB_GEMM_TRACE
        if (p.trace && threadIdx.x == 0) p.trace[(size_t)lin * 16 + 9] = __builtin_amdgcn_s_memrealtime();
#endif
        const bool to_seg = p.c_seg != nullptr && dst == p.C;   // the final output goes to the segments' own buffers
        constexpr int LPR = BN / 8;                  // lanes per row (16 bytes each)
        constexpr int RPI = 64 / LPR;                // rows per store instruction
        const int col = (lane % LPR) * 8;
#pragma unroll 4
        for (int r = wave * RPI + lane / LPR; r < BM; r += (NT / 64) * RPI) {
            const int m = m0 + r, n = n0 + col;
            if (m < p.M && n < p.N) {
                bf16* rowp = dst + (size_t)m * p.N;
                if (to_seg) {
                    const int s = seg_of_row(p.off, seg_lo, seg_hi, m);
                    rowp = p.c_seg[s] + (size_t)(m - p.off[s]) * p.N;
                }
                *reinterpret_cast<uint4*>(rowp + n) = *reinterpret_cast<const uint4*>(smem + r * CP + col * 2);
            }
        }
    };

    // ---- optional store of the pre-adapter output (accumulator + bias, before the LoRA term)
    if (p.Cbase) {
        stage_out(p.Cbase, false);
        __syncthreads();                             // LDS is reused by the LoRA tiles below
    }

    // ---- LoRA term: extra K-steps per LoRA segment that meets this row tile
    if (p.ext) {
        for (int s = seg_lo; s <= seg_hi; ++s) {
            const SegDesc sd = p.seg[s];
            const int r_lo = max(p.off[s], m0), r_hi = min(min(p.off[s + 1], m0 + BM), p.M);
            if (sd.kind != KIND_LORA || r_hi <= r_lo) continue;      // uniform over the workgroup
            const int kext = 2 * sd.rpad;                           // value half, then residual half
            for (int kc0 = 0; kc0 < kext; kc0 += BK) {
                // activation-side tile: rows of this segment only, others zero
#pragma unroll
                for (int i = 0; i < CA; ++i) {
                    const int c = tid + i * NT, row = c >> 3, kc = c & 7, m = m0 + row;
                    const bool ok = m >= r_lo && m < r_hi && (kc0 + kc * 8) < kext;
                    ra[i] = ld_global_16(p.ext + (size_t)(ok ? m : 0) * p.ext_pitch + kc0 + kc * 8, ok);
                }
                // adapter-side tile
#pragma unroll
                for (int i = 0; i < CB; ++i) {
                    const int c = tid + i * NT;
                    if constexpr (!NN) {       // B_i [N][rank], rank-contiguous
                        const int row = c >> 3, kc = c & 7, n = n0 + row;
                        const int pk = kc0 + kc * 8, pp = pk >= sd.rpad ? pk - sd.rpad : pk;   // both halves meet the same B_i
                        uint4 v = make_uint4(0u, 0u, 0u, 0u);
                        if (n < p.N && pk < kext && pp < sd.rank) {
                            const bf16* src = sd.B + (size_t)n * sd.rank + pp;
                            if ((sd.rank & 7) == 0) {
                                v = *reinterpret_cast<const uint4*>(src);
                            } else {
                                unsigned short e[8];
#pragma unroll
                                for (int q = 0; q < 8; ++q)
                                    e[q] = (pp + q < sd.rank) ? reinterpret_cast<const unsigned short*>(src)[q] : (unsigned short)0;
                                v.x = e[0] | ((unsigned)e[1] << 16); v.y = e[2] | ((unsigned)e[3] << 16);
                                v.z = e[4] | ((unsigned)e[5] << 16); v.w = e[6] | ((unsigned)e[7] << 16);
                            }
                        }
                        rb[i] = v;
                    } else {                   // A_i [rank][N], N-contiguous
                        const int krow = c / (BN / 8), nc = c % (BN / 8), n = n0 + nc * 8;
                        const int pk = kc0 + krow, pp = pk >= sd.rpad ? pk - sd.rpad : pk;
                        const bool ok = pk < kext && pp < sd.rank && n < p.N;
                        rb[i] = ld_global_16(sd.A + (size_t)(ok ? pp : 0) * p.N + (ok ? n : 0), ok);
                    }
                }
                lds_store(0);
                __syncthreads();
                compute(min(BK, kext - kc0) >> 4);
                __syncthreads();
            }
        }
    }

#ifdef SYMB_GEMM_TRACE
    if (p.trace && threadIdx.x == 0) p.trace[(size_t)lin * 16 + 4] = __builtin_amdgcn_s_memrealtime();
#endif
    // ---- final output: bias, IA3 scale, one rounding, whole-row stores
    stage_out(p.C, p.epi_ia3 != 0);          // (the noise effect, if any, comes off here; Cbase is never asked for then)
#ifdef SYMB_GEMM_TRACE
    if (p.trace && threadIdx.x == 0) p.trace[(size_t)lin * 16 + 7] = __builtin_amdgcn_s_memrealtime();
    __builtin_amdgcn_s_waitcnt(0);
    if (p.trace && threadIdx.x == 0) { p.trace[(size_t)lin * 16 + 3] = __builtin_amdgcn_s_memrealtime(); p.trace[(size_t)lin * 16 + 6] = __builtin_readcyclecounter(); }
#endif
}

}  // namespace symb
