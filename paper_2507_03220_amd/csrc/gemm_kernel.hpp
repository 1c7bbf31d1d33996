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
// Tiling (gfx950): one workgroup owns a BM x BN tile of C; K is walked in steps of 64
// through double-buffered LDS; WGM x WGN wavefronts of 64 lanes each own a
// (BM/WGM) x (BN/WGN) sub-tile as 32x32 blocks of v_mfma_f32_32x32x16_bf16.  The MFMA
// is issued as (weight fragment, activation fragment), so a lane ends up holding, for
// one row m, runs of 4 consecutive n: rows keep their own segment in the epilogue and
// the store is 8 bytes per lane.
#pragma once
#include "symb_device.hpp"

namespace symb {

struct GemmParams {
    const bf16* Aop;            // [M][K]
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
    int epi_ia3;                // forward: scale rows of IA3 segments by l_i[n]
    double timing_flops;        // host bookkeeping for the measurement hook; unused on the device
};

constexpr int GEMM_BK = 64;

// 16-byte chunk swizzle of a K-contiguous tile row (8 chunks of 8 bf16 per row).
__device__ __forceinline__ int swz_row(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int BM, int BN, int WGM, int WGN, bool NN>
struct GemmTile {
    static constexpr int NT = WGM * WGN * 64;
    static constexpr int BK = GEMM_BK;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int MB = WTM / 32, NB = WTN / 32;
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int SMEM = 2 * (A_BYTES + B_BYTES);
    static constexpr int CA = BM * 8 / NT, CB = BN * 8 / NT;   // 16-byte chunks per thread per K-step
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
    const int per_xcd = (total + 7) >> 3;
    const int lin = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (lin >= total || (int)(blockIdx.x >> 3) >= per_xcd) return;
    const int width = p.group_m * p.num_n_tiles;
    const int first_m = (lin / width) * p.group_m;
    const int gsz = min(p.num_m_tiles - first_m, p.group_m);
    const int tm = first_m + (lin % width) % gsz;
    const int tn = (lin % width) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / WGN) * TT::WTM, wn0 = (wave % WGN) * TT::WTN;

    floatx16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- per-thread global load slots.  Chunk i of a thread sits NT/8 rows (K-contiguous tiles)
    // or NT/(BN/8) k-rows (N-contiguous weight tile) below chunk 0, in the same 16-byte column, so
    // one pointer and one LDS offset per operand are enough (the swizzles repeat every 16 rows).
    constexpr int RSTEP = NT / 8;                 // row step between a thread's chunks, K-contiguous tile
    constexpr int KSTEP = NT / (BN / 8);          // k-row step, N-contiguous tile
    static_assert(RSTEP % 16 == 0 && (!NN || KSTEP % 4 == 0), "chunk stride must preserve the LDS swizzle");
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;
    const bf16* a_base = p.Aop + (size_t)(m0 + lrow) * p.K + lkc;
    const int a_lds0 = lds_off_kmajor(lrow, tid & 7);
    const bf16* b_base;
    int b_lds0;
    const int nn_k = tid / (BN / 8), nn_nc = tid % (BN / 8);
    const bool nn_ok = (n0 + nn_nc * 8) < p.N;
    if constexpr (!NN) {
        b_base = p.Bop + (size_t)(n0 + lrow) * p.K + lkc;
        b_lds0 = a_lds0;
    } else {
        b_base = p.Bop + (size_t)nn_k * p.N + (nn_ok ? (n0 + nn_nc * 8) : 0);
        b_lds0 = lds_off_nmajor<BN>(nn_k, nn_nc);
    }

    uint4 ra[CA], rb[CB];
    auto gload = [&](int k0) {
        const bool kok = (k0 + lkc) < p.K;
#pragma unroll
        for (int i = 0; i < CA; ++i)
            ra[i] = ld_global_16(a_base + (size_t)i * RSTEP * p.K + k0, kok && (m0 + lrow + i * RSTEP) < p.M);
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            if constexpr (!NN)
                rb[i] = ld_global_16(b_base + (size_t)i * RSTEP * p.K + k0, kok && (n0 + lrow + i * RSTEP) < p.N);
            else
                rb[i] = ld_global_16(b_base + (size_t)(k0 + i * KSTEP) * p.N, nn_ok && (k0 + nn_k + i * KSTEP) < p.K);
        }
    };
    auto lds_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < CA; ++i) *reinterpret_cast<uint4*>(sA + buf * TT::A_BYTES + a_lds0 + i * RSTEP * 128) = ra[i];
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            if constexpr (!NN) *reinterpret_cast<uint4*>(sB + buf * TT::B_BYTES + b_lds0 + i * RSTEP * 128) = rb[i];
            else *reinterpret_cast<uint4*>(sB + buf * TT::B_BYTES + b_lds0 + i * KSTEP * (BN * 2)) = rb[i];
        }
    };
    auto compute = [&](int buf, int nks) {
        const unsigned char* bufA = sA + buf * TT::A_BYTES;
        const unsigned char* bufB = sB + buf * TT::B_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks < nks) {
                bf16x8 xa[MB], wb[NB];
#pragma unroll
                for (int i = 0; i < MB; ++i)
                    xa[i] = lds_read_frag_kmajor(bufA, wm0 + i * 32 + (lane & 31), ks * 2 + (lane >> 5));
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    if constexpr (!NN) wb[j] = lds_read_frag_kmajor(bufB, wn0 + j * 32 + (lane & 31), ks * 2 + (lane >> 5));
                    else wb[j] = lds_read_frag_nmajor<BN>(bufB, wn0 + j * 32, ks * 16, lane);
                }
#pragma unroll
                for (int i = 0; i < MB; ++i)
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wb[j], xa[i], acc[i][j], 0, 0, 0);
            }
        }
    };

    // ---- main loop over K: global -> registers -> LDS, double buffered
    const int KT = (p.K + BK - 1) / BK;
    gload(0);
    lds_store(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < KT) gload((kt + 1) * BK);
        compute(cur, BK / 16);
        if (kt + 1 < KT) lds_store(cur ^ 1);
        __syncthreads();
    }

    // ---- bias, optional store of the pre-adapter output
    const int seg_lo = p.tile_seg_lo[tm], seg_hi = p.tile_seg_hi[tm];
    auto for_each_quad = [&](auto&& fn) {
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
    if (p.bias) {
        for_each_quad([&](int i, int j, int rg, int, int n) {
            if (n < p.N) {
                const uint2 bv = *reinterpret_cast<const uint2*>(p.bias + n);
                acc[i][j][rg * 4 + 0] += bf16_bits_to_f32((unsigned short)(bv.x & 0xffffu));
                acc[i][j][rg * 4 + 1] += bf16_bits_to_f32((unsigned short)(bv.x >> 16));
                acc[i][j][rg * 4 + 2] += bf16_bits_to_f32((unsigned short)(bv.y & 0xffffu));
                acc[i][j][rg * 4 + 3] += bf16_bits_to_f32((unsigned short)(bv.y >> 16));
            }
        });
    }
    if (p.Cbase) {
        for_each_quad([&](int i, int j, int rg, int m, int n) {
            if (m < p.M && n < p.N) {
                uint2 o;
                o.x = pack2_bf16(acc[i][j][rg * 4 + 0], acc[i][j][rg * 4 + 1]);
                o.y = pack2_bf16(acc[i][j][rg * 4 + 2], acc[i][j][rg * 4 + 3]);
                *reinterpret_cast<uint2*>(p.Cbase + (size_t)m * p.N + n) = o;
            }
        });
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
                compute(0, min(BK, kext - kc0) >> 4);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: IA3 scale of each row's own segment, one rounding to bf16, 8-byte stores
    for_each_quad([&](int i, int j, int rg, int m, int n) {
        if (m < p.M && n < p.N) {
            float v0 = acc[i][j][rg * 4 + 0], v1 = acc[i][j][rg * 4 + 1];
            float v2 = acc[i][j][rg * 4 + 2], v3 = acc[i][j][rg * 4 + 3];
            if (p.epi_ia3) {
                const int s = seg_of_row(p.off, seg_lo, seg_hi, m);
                if (p.seg[s].kind == KIND_IA3) {
                    const uint2 lv = *reinterpret_cast<const uint2*>(p.seg[s].A + n);
                    v0 *= bf16_bits_to_f32((unsigned short)(lv.x & 0xffffu));
                    v1 *= bf16_bits_to_f32((unsigned short)(lv.x >> 16));
                    v2 *= bf16_bits_to_f32((unsigned short)(lv.y & 0xffffu));
                    v3 *= bf16_bits_to_f32((unsigned short)(lv.y >> 16));
                }
            }
            uint2 o;
            o.x = pack2_bf16(v0, v1);
            o.y = pack2_bf16(v2, v3);
            *reinterpret_cast<uint2*>(p.C + (size_t)m * p.N + n) = o;
        }
    });
}

}  // namespace symb
