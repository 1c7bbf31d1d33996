// HBM-bound kernels around the base GEMM: LoRA shrink (Hs = s X A^T), its backward twin
// (dH = s dY B), the per-segment parameter gradients (dA, dB, dl) and the IA3 row scale
// of dY.  All of them walk segment-aligned row chunks from a host-built work list, so a
// chunk never mixes two clients.
#pragma once
#include <type_traits>

#include "symb_device.hpp"

namespace symb {

// One unit of row work: rows [row0, row0 + nrows) of segment `seg` (nrows <= chunk size).
struct RowChunk {
    int32_t seg, row0, nrows, pad;
};

// -------------------------------------------------------------------------------------------
// Skinny projection:  out[t][p] = s_i * sum_k L[t][k] * R_i[p][k],  p < rpad_i, stored as a bf16
// value plus a bf16 residual (out[t][rpad_i + p])
//   forward shrink : L = X  [T][K=d_in],  R_i = A_i  [r][d_in]
//   backward dH    : L = dY [T][K=d_out], R_i = B_i^T packed [rpad][d_out] (see pack kernel)
// A workgroup owns 32 rows; its 4 wavefronts split K in interleaved slices, bring the rows in
// through LDS (see SkinnyStage below), take the adapter rows from L2, and meet in LDS for the
// final sum.  RB = max rank blocks of 16.
// -------------------------------------------------------------------------------------------
struct SkinnyParams {
    const bf16* L;            // [T][K]
    bf16* out;                // [T][out_pitch], out_pitch >= 2 * rpad_i
    int K, out_pitch;
    const RowChunk* chunks;   // device
    const SegDesc* seg;       // device
    const bf16* packed;       // backward: base of packed B^T area, else null
    const int64_t* packed_off;// backward: element offset of segment i's [rpad][K] block
    int use_packed;
    const bf16* const* L_seg; // device [S] or null: rows of segment i start at L_seg[i] instead of L + off[i] * K
    const int32_t* off;       // device [S+1] (read only with L_seg)
};

constexpr int SKINNY_BLKS = 2;                         // 16-row MFMA blocks per wavefront
constexpr int SKINNY_ROWS = 16 * SKINNY_BLKS;          // rows per workgroup

// The skinny kernel's row stream.  A lane of an MFMA operand holds 16 bytes of one row, so fragment
// loads straight from global memory touch 16 cache lines per 16 lanes, 16 bytes of each; the
// memory pipeline then runs at a fraction of what whole-line requests reach.  Here every wavefront
// brings its K slices (SKINNY_ROWS rows x SK elements) in through LDS DMA, whole rows of the slice
// per request, into NBUF buffers of its own (no workgroup barrier in the loop), and reads the
// fragments from LDS.  The 16-byte chunks of a row are stored at chunk ^ f(row), so the 16 rows a
// fragment read touches fall on different banks.  The adapter rows of a slice (from L2) come the same
// way, into one more buffer.  Measured on 1.5 GB inputs: 4.0 -> 5.0 TB/s; 128-element slices are best
// at rank <= 16, 64-element ones above (LDS for the adapter rows); a third buffer or a third workgroup
// per CU changes nothing.
template <int RB, int NBUF_ = 2, bool RDEEP_ = false>
struct SkinnyStage {
    static constexpr int SK = RB >= 2 ? 64 : 128;         // K elements per slice
    static constexpr int NBUF = NBUF_;                    // slices a wavefront keeps in LDS
    static constexpr bool RDEEP = RDEEP_;                 // the adapter rows are requested with their slice, NBUF deep as well
    static constexpr int ROW_BYTES = SK * 2;
    static constexpr int LPR = ROW_BYTES / 16;            // lanes (16-byte chunks) per row
    static constexpr int RPI = 64 / LPR;                  // rows per DMA request of one wavefront
    static constexpr int DPS = SKINNY_ROWS / RPI;         // DMA requests per slice
    static constexpr int SLICE = SKINNY_ROWS * ROW_BYTES;
    static constexpr int RSLICE = RB * 16 * ROW_BYTES;    // the adapter rows of one slice (one buffer)
    static constexpr int WAVE_BYTES = NBUF * SLICE + (RDEEP ? NBUF : 1) * RSLICE;
    static constexpr int BYTES = 4 * WAVE_BYTES;
    static_assert(SK == 64 || SK == 128, "a row of a slice is one or two 128-byte lines");
    __device__ static constexpr int swz(int r) { return (r / (16 / LPR)) & (LPR - 1); }
};
typedef __attribute__((address_space(1))) void glb_void_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// 16 bytes from global memory.  Said explicitly: a pointer that was itself loaded from memory (an
// adapter's address in its descriptor) is generic to the compiler, and a generic load counts on both
// memory counters, which forces full waits around it.
__device__ __forceinline__ u32x4 ld_glb16(const bf16* p) {
    return *reinterpret_cast<const __attribute__((address_space(1))) u32x4*>((const __attribute__((address_space(1))) bf16*)p);
}

// One wavefront's share of K for a chunk whose segment uses NB rank blocks (compile time, so that the
// loop holds no conditional load: the compiler's wait counts for the adapter rows are then exact).
// lrow / rrow point at the lane's first 8 elements (row start + kq*8); src[i] at the 16 bytes this
// lane brings in with DMA request i of a slice (at k = 0); wbuf = this wavefront's slice buffers.
template <int RB, int NB, class ST = SkinnyStage<RB>>
__device__ __forceinline__ void skinny_stream(const bf16* (&lrow)[SKINNY_BLKS], const bf16* (&rrow)[RB], const bool (&r_ok)[RB],
                                              const bf16* (&src)[ST::DPS], const bf16* rbase, int rrows,
                                              unsigned char* wbuf, int K, int wave, int lane, floatx4 (&acc)[SKINNY_BLKS][RB]) {
    constexpr int NH = ST::SK / 32;                      // MFMA k-steps per slice
    constexpr int NRD = NB * 16 / ST::RPI;               // DMA requests for the adapter rows of a slice
    const int trow = lane & 15, kq = lane >> 4;
    unsigned char* const rbuf = wbuf + ST::NBUF * ST::SLICE;
    unsigned foff[SKINNY_BLKS][NH], roff[NB][NH];        // fragment (b, h) / (j, h) of this lane within a slice buffer
#pragma unroll
    for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int b = 0; b < SKINNY_BLKS; ++b) {
            const int r = b * 16 + trow;
            foff[b][h] = (unsigned)(size_t)wbuf + (unsigned)(r * ST::ROW_BYTES + (((h * 4 + kq) ^ ST::swz(r)) * 16));
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int r = j * 16 + trow;
            roff[j][h] = (unsigned)(size_t)rbuf + (unsigned)(r * ST::ROW_BYTES + (((h * 4 + kq) ^ ST::swz(r)) * 16));
        }
    }
    // The adapter rows (from L2) come in by LDS DMA as well, whole row pieces per request: fragment loads
    // straight from global memory are 64-byte pieces of 16 rows each, twice the requests for the bytes.
    // Rows past the adapter's last are read from row 0 and count as zero (r_ok).
    const bf16* rsrc[NRD];
#pragma unroll
    for (int i = 0; i < NRD; ++i) {
        const int r = i * ST::RPI + lane / ST::LPR;
        rsrc[i] = rbase + (size_t)(r < rrows ? r : 0) * K + (((lane % ST::LPR) ^ ST::swz(r)) * 8);
    }
    auto dma = [&](int buf, int k) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < ST::DPS; ++i)
            __builtin_amdgcn_global_load_lds((glb_void_t*)(src[i] + k), (lds_void_t*)(wbuf + buf * ST::SLICE + i * 1024), 16, 0, 0);
    };
    auto dma_r = [&](int buf, int k) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NRD; ++i)
            __builtin_amdgcn_global_load_lds((glb_void_t*)(rsrc[i] + k), (lds_void_t*)(rbuf + (ST::RDEEP ? buf * ST::RSLICE : 0) + i * 1024), 16, 0, 0);
    };
    // The fragment reads are assembly statements with a wait of their own: while an LDS DMA request is in
    // flight the compiler makes every load result it can see wait for all memory traffic of the
    // wavefront, the slice requested ahead included.  Each result is tied ("+v") to the wait that
    // covers it, so no use can move in front of that wait.  mul() returns with its LDS reads
    // complete: both buffers it read may be requested again.
    auto mul = [&](int buf) __attribute__((always_inline)) {
        u32x4 lv[SKINNY_BLKS][NH], rv[NB][NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) {
#pragma unroll
            for (int b = 0; b < SKINNY_BLKS; ++b) asm volatile("ds_read_b128 %0, %1" : "=v"(lv[b][h]) : "v"(foff[b][h] + buf * ST::SLICE));
#pragma unroll
            for (int j = 0; j < NB; ++j) asm volatile("ds_read_b128 %0, %1" : "=v"(rv[j][h]) : "v"(roff[j][h] + (ST::RDEEP ? buf * ST::RSLICE : 0)));
        }
        asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
#pragma unroll
        for (int h = 0; h < NH; ++h) {
#pragma unroll
            for (int b = 0; b < SKINNY_BLKS; ++b) asm volatile("" : "+v"(lv[b][h]));
#pragma unroll
            for (int j = 0; j < NB; ++j) asm volatile("" : "+v"(rv[j][h]));
        }
#pragma unroll
        for (int h = 0; h < NH; ++h)
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const bf16x8 rf = __builtin_bit_cast(bf16x8, r_ok[j] ? rv[j][h] : u32x4{0u, 0u, 0u, 0u});
#pragma unroll
                for (int b = 0; b < SKINNY_BLKS; ++b)
                    acc[b][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rf, __builtin_bit_cast(bf16x8, lv[b][h]), acc[b][j], 0, 0, 0);
            }
    };
    // ---- full slices of this wavefront: k = wave * SK + 4 SK s, s < ns, through LDS.  Slices 0 .. np-1
    // are requested up front; iteration s requests slice s + np (while there is one) into the buffer
    // iteration s - 1 has finished reading, after the adapter rows of slice s: the memory counter
    // retires in order, so the wait for slice s and its adapter rows leaves exactly the newest slice's
    // DPS requests in flight.
    int k0 = wave * ST::SK;
    const int ns = K >= k0 + ST::SK ? (K - k0 - ST::SK) / (4 * ST::SK) + 1 : 0;
    const int np = ns < ST::NBUF - 1 ? ns : ST::NBUF - 1;
    for (int d = 0; d < np; ++d) {
        dma(d, k0 + d * 4 * ST::SK);
        if constexpr (ST::RDEEP) dma_r(d, k0 + d * 4 * ST::SK);
    }
    int cur = 0, nxt = np;                               // buffer of slice s, of slice s + np
    int s = 0;
    for (; s + np < ns; ++s) {
        if constexpr (ST::RDEEP) {                       // slice and adapter rows together, NBUF - 1 of them in flight
            dma(nxt, k0 + np * 4 * ST::SK);
            dma_r(nxt, k0 + np * 4 * ST::SK);
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"((ST::NBUF - 1) * (ST::DPS + NRD)) : "memory");
        } else {
            dma_r(0, k0);
            dma(nxt, k0 + np * 4 * ST::SK);
            asm volatile("s_waitcnt vmcnt(%0)" : : "n"(ST::DPS) : "memory");
        }
        mul(cur);
        cur = cur + 1 == ST::NBUF ? 0 : cur + 1;
        nxt = nxt + 1 == ST::NBUF ? 0 : nxt + 1;
        k0 += 4 * ST::SK;
    }
    for (; s < ns; ++s) {                                // the last np slices: nothing left to request
        if constexpr (!ST::RDEEP) dma_r(0, k0);
        asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
        mul(cur);
        cur = cur + 1 == ST::NBUF ? 0 : cur + 1;
        k0 += 4 * ST::SK;
    }
    // ---- the slice that crosses the end of K: masked fragments straight from global memory
    if (k0 < K) {
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const bool kok = (k0 + h * 32 + kq * 8) < K;
            u32x4 lv[SKINNY_BLKS];
#pragma unroll
            for (int b = 0; b < SKINNY_BLKS; ++b) lv[b] = kok ? ld_glb16(lrow[b] + k0 + h * 32) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const u32x4 rv = (kok && r_ok[j]) ? ld_glb16(rrow[j] + k0 + h * 32) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int b = 0; b < SKINNY_BLKS; ++b)
                    acc[b][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, rv), __builtin_bit_cast(bf16x8, lv[b]), acc[b][j], 0, 0, 0);
            }
        }
    }
}

// Calls skinny_stream<RB, nb> for the run-time nb in 1..RB.
template <int RB, class ST, int NB = 1, typename... Args>
__device__ __forceinline__ void skinny_stream_dispatch(int nb, Args&&... args) {
    if (nb == NB) skinny_stream<RB, NB, ST>(args...);
    else if constexpr (NB < RB) skinny_stream_dispatch<RB, ST, NB + 1>(nb, args...);
}

// DEEP: three buffers with the adapter rows beside each slice, two slices in flight per wavefront.  For
// launches of few chunks, where a workgroup has a compute unit to itself and its time is the chain of
// memory latencies along K rather than bandwidth.
template <int RB, bool DEEP = false>
__global__ void __launch_bounds__(256)
symb_skinny_kernel(const SkinnyParams p) {
    using ST = SkinnyStage<RB, DEEP ? 3 : 2, DEEP>;
    constexpr int RED_BYTES = 3 * SKINNY_ROWS * (RB * 16 + 4) * 4;
    // slice buffers of the 4 wavefronts; afterwards the partial sums of wavefronts 1..3
    __shared__ __align__(16) unsigned char smem[ST::BYTES > RED_BYTES ? ST::BYTES : RED_BYTES];
    float (*red)[SKINNY_ROWS][RB * 16 + 4] = reinterpret_cast<float (*)[SKINNY_ROWS][RB * 16 + 4]>(smem);
    const RowChunk ch = p.chunks[blockIdx.x];
    const SegDesc sd = p.seg[ch.seg];
    const int nb = sd.rpad >> 4;                         // rank blocks in use (uniform), 1..RB
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int trow = lane & 15, kq = lane >> 4;
    // rows past the chunk are clamped onto its last row; their results are never stored
    const bf16* lrow[SKINNY_BLKS];
    const bf16* const lbase = p.L_seg ? p.L_seg[ch.seg] - (size_t)p.off[ch.seg] * p.K : p.L;
#pragma unroll
    for (int b = 0; b < SKINNY_BLKS; ++b) lrow[b] = lbase + (size_t)(ch.row0 + min(b * 16 + trow, ch.nrows - 1)) * p.K + kq * 8;
    const bf16* src[ST::DPS];
#pragma unroll
    for (int i = 0; i < ST::DPS; ++i) {
        const int r = i * ST::RPI + lane / ST::LPR;
        src[i] = lbase + (size_t)(ch.row0 + min(r, ch.nrows - 1)) * p.K + (((lane % ST::LPR) ^ ST::swz(r)) * 8);
    }
    const bf16* rbase = p.use_packed ? (p.packed + p.packed_off[ch.seg]) : sd.A;
    const int rrows = p.use_packed ? sd.rpad : sd.rank;  // valid adapter rows; the rest count as zero
    const bf16* rrow[RB];
    bool r_ok[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        r_ok[j] = (j * 16 + trow) < rrows;
        rrow[j] = rbase + (size_t)(r_ok[j] ? (j * 16 + trow) : 0) * p.K + kq * 8;
    }

    floatx4 acc[SKINNY_BLKS][RB];
#pragma unroll
    for (int b = 0; b < SKINNY_BLKS; ++b)
#pragma unroll
        for (int j = 0; j < RB; ++j) acc[b][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    skinny_stream_dispatch<RB, ST>(nb, lrow, rrow, r_ok, src, rbase, rrows, smem + wave * ST::WAVE_BYTES, p.K, wave, lane, acc);
    __syncthreads();                                     // every wavefront is done with its slice buffers
    // lane holds out[t = b*16 + trow][p = j*16 + 4*kq + q]
    if (wave > 0) {
#pragma unroll
        for (int b = 0; b < SKINNY_BLKS; ++b)
#pragma unroll
            for (int j = 0; j < RB; ++j)
                if (j < nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) red[wave - 1][b * 16 + trow][j * 16 + kq * 4 + q] = acc[b][j][q];
    }
    __syncthreads();
    // One row of `out` holds, for its own segment, rpad values rounded to bf16 followed by the
    // rpad rounding residuals (also bf16): value + residual carries ~16 significand bits on.
    if (wave == 0) {
#pragma unroll
        for (int b = 0; b < SKINNY_BLKS; ++b) {
            const int t = b * 16 + trow;
            if (t < ch.nrows) {
                bf16* row = p.out + (size_t)(ch.row0 + t) * p.out_pitch;
#pragma unroll
                for (int j = 0; j < RB; ++j)
                    if (j < nb) {
                        const int pp = j * 16 + kq * 4;
                        float v[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            v[q] = sd.scale * (acc[b][j][q] + red[0][t][pp + q] + red[1][t][pp + q] + red[2][t][pp + q]);
                        const unsigned h01 = pack2_bf16(v[0], v[1]), h23 = pack2_bf16(v[2], v[3]);
                        uint2 hi2, lo2;
                        hi2.x = h01;
                        hi2.y = h23;
                        lo2.x = pack2_bf16(v[0] - bf16_bits_to_f32((unsigned short)(h01 & 0xffffu)), v[1] - bf16_bits_to_f32((unsigned short)(h01 >> 16)));
                        lo2.y = pack2_bf16(v[2] - bf16_bits_to_f32((unsigned short)(h23 & 0xffffu)), v[3] - bf16_bits_to_f32((unsigned short)(h23 >> 16)));
                        *reinterpret_cast<uint2*>(row + pp) = hi2;
                        *reinterpret_cast<uint2*>(row + sd.rpad + pp) = lo2;
                    }
            }
        }
    }
}

// Transposing LDS read of an MFMA fragment whose k axis runs down the rows of a column-contiguous tile.
__device__ __forceinline__ bf16x8 lds_read_tr_16x32(const unsigned char* base, int pitch_bytes, int col0, int lane) {
    // tile [32 t][cols] (column-contiguous); returns for lane l: column col0 + (l & 15), t = 8*(l >> 4) + 0..7
    const int g = lane >> 4, jj = lane & 15;
    const unsigned char* p0 = base + (g * 8 + (jj >> 2)) * pitch_bytes + (col0 + ((jj & 3) << 2)) * 2;
    typedef __attribute__((address_space(3))) shortx4 lds_s4;
    shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p0));
    shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)(p0 + 4 * pitch_bytes));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short shortx8;
    shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// -------------------------------------------------------------------------------------------
// Calls of at most 16 rows (decode steps of inference clients, the input gradient of a short
// fine-tuning segment; Sec. 3.6 / 3.7: such requests interleave with the large ones per layer).
// A tiled GEMM launches too few workgroups for so few rows to stream the weight at HBM speed, so
// these calls take kernels of their own that read the weight exactly once:
//   C[t][n] = sum_k A[t][k] * Wop[n][k]   (the weight read K-contiguous: symb_rowgemv_kernel)
//   C[t][n] = sum_k A[t][k] * Wop[k][n]   (the weight read N-contiguous: symb_colgemv_kernel,
//                                          partial sums over K ranges, symb_small_finish_kernel)
// A is flat [T][K] (per-client buffers and rows that need a scale are gathered into the workspace
// first: a few KiB).  Every (row, column) result is finished with its row's own adapter by
// small_epilogue: same arithmetic as the tiled path (fp32 accumulation, Hs / dH as value +
// residual, one rounding to bf16).
// -------------------------------------------------------------------------------------------
struct SmallEpilogue {
    bf16* C;                  // [T][N] flat, or null with c_seg
    bf16* Cbase;              // [T][N] or null: the value (+ bias) before the adapter term
    bf16* const* c_seg;       // device [S] or null: row t of segment i goes to c_seg[i] + (t - off[i]) * N
    const bf16* bias;         // [N] or null
    int N, T, S;
    const int32_t* off;       // device [S+1]
    const SegDesc* seg;       // device [S]
    const bf16* ext;          // [T][ext_pitch]: Hs (forward) or dH (input gradient); null = no LoRA term
    int ext_pitch;
    int backward;             // 0: forward (+ Hs B_i[n][.], * IA3 l[n], - noise effect); 1: input gradient (+ dH A_i[.][n], * IA3_IN l[n])
    int lora_term;            // 0: no LoRA term at all (base-only input gradient)
    const NoiseDesc* neff;    // device [S] or null (forward only)
};

// Finishes C[t][n] from its fp32 sum v; s = the row's segment.
__device__ __forceinline__ void small_epilogue(const SmallEpilogue& e, int t, int n, int s, float v) {
    if (e.bias) v += bf16_bits_to_f32(reinterpret_cast<const unsigned short*>(e.bias)[n]);
    if (e.Cbase) reinterpret_cast<unsigned short*>(e.Cbase)[(size_t)t * e.N + n] = (unsigned short)(pack2_bf16(v, 0.f) & 0xffffu);
    const SegDesc sd = e.seg[s];
    if (sd.kind == KIND_LORA && e.lora_term) {
        const unsigned short* hrow = reinterpret_cast<const unsigned short*>(e.ext) + (size_t)t * e.ext_pitch;
        float u = 0.f;
        if (!e.backward) {
            const unsigned short* brow = reinterpret_cast<const unsigned short*>(sd.B) + (size_t)n * sd.rank;
            for (int q = 0; q < sd.rank; ++q)
                u += (bf16_bits_to_f32(hrow[q]) + bf16_bits_to_f32(hrow[sd.rpad + q])) * bf16_bits_to_f32(brow[q]);
        } else {
            const unsigned short* acol = reinterpret_cast<const unsigned short*>(sd.A) + n;
            for (int q = 0; q < sd.rank; ++q)
                u += (bf16_bits_to_f32(hrow[q]) + bf16_bits_to_f32(hrow[sd.rpad + q])) * bf16_bits_to_f32(acol[(size_t)q * e.N]);
        }
        v += u;
    } else if (sd.kind == (e.backward ? KIND_IA3_IN : KIND_IA3) && (e.lora_term || !e.backward)) {
        v *= bf16_bits_to_f32(reinterpret_cast<const unsigned short*>(sd.A)[n]);
    }
    if (e.neff) {
        const NoiseDesc nd = e.neff[s];
        if (nd.ptr) v -= bf16_bits_to_f32(reinterpret_cast<const unsigned short*>(nd.ptr)[(size_t)(nd.rows == 1 ? 0 : t - e.off[s]) * e.N + n]);
    }
    unsigned short* out = e.c_seg ? reinterpret_cast<unsigned short*>(e.c_seg[s]) + (size_t)(t - e.off[s]) * e.N
                                  : reinterpret_cast<unsigned short*>(e.C) + (size_t)t * e.N;
    out[n] = (unsigned short)(pack2_bf16(v, 0.f) & 0xffffu);
}

// Segment of each of the (at most 16 RB) rows, into LDS.
__device__ __forceinline__ void small_row_segments(const SmallEpilogue& e, int* srow, int nrows_max) {
    if ((int)threadIdx.x < nrows_max) {
        int s = 0;
        if ((int)threadIdx.x < e.T) {
            while (s + 1 < e.S && (int)threadIdx.x >= e.off[s + 1]) ++s;
        }
        srow[threadIdx.x] = s;
    }
}

// ---- weight read K-contiguous.  A workgroup owns 32 output columns: it streams those 32 rows of the
// weight once (the 4 wavefronts split K; through LDS, like the skinny kernel's rows) and multiplies them
// with all rows of A (from L2).  RB = row blocks of 16 (T <= 16 RB; the library uses RB = 1: beyond 16
// rows the tiled kernel with its K-split is faster).
struct RowGemvParams {
    const bf16* W;            // [N][K]
    const bf16* X;            // [T][K]
    int K;
    SmallEpilogue epi;
};

template <int RB>
__global__ void __launch_bounds__(256)
symb_rowgemv_kernel(const RowGemvParams p) {
    using ST = SkinnyStage<RB, 3, true>;                 // W rows and X rows of a slice together, two slices ahead:
    // with one workgroup per 32 columns there are few wavefronts, each must keep a lot in flight
    __shared__ __align__(16) unsigned char stage[ST::BYTES];
    __shared__ float red[3][SKINNY_ROWS][RB * 16 + 4];   // partial sums of wavefronts 1..3; red[0] then holds the totals
    __shared__ int srow[RB * 16];                        // segment of each row
    static_assert(SKINNY_BLKS == 2, "a workgroup owns 32 columns");
    const int N = p.epi.N, T = p.epi.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int trow = lane & 15, kq = lane >> 4;
    const int n0 = blockIdx.x * SKINNY_ROWS;
    small_row_segments(p.epi, srow, RB * 16);
    // columns past N are clamped onto the last one; their results are never stored
    const bf16* lrow[SKINNY_BLKS];
#pragma unroll
    for (int b = 0; b < SKINNY_BLKS; ++b) lrow[b] = p.W + (size_t)min(n0 + b * 16 + trow, N - 1) * p.K + kq * 8;
    const bf16* rrow[RB];
    bool r_ok[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        r_ok[j] = (j * 16 + trow) < T;
        rrow[j] = p.X + (size_t)(r_ok[j] ? (j * 16 + trow) : 0) * p.K + kq * 8;
    }
    floatx4 acc[SKINNY_BLKS][RB];
#pragma unroll
    for (int b = 0; b < SKINNY_BLKS; ++b)
#pragma unroll
        for (int j = 0; j < RB; ++j) acc[b][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    const bf16* src[ST::DPS];                            // this lane's 16 bytes of DMA request i of a slice (at k = 0)
#pragma unroll
    for (int i = 0; i < ST::DPS; ++i) {
        const int r = i * ST::RPI + lane / ST::LPR;
        src[i] = p.W + (size_t)min(n0 + r, N - 1) * p.K + (((lane % ST::LPR) ^ ST::swz(r)) * 8);
    }
    skinny_stream<RB, RB, ST>(lrow, rrow, r_ok, src, p.X, T, stage + wave * ST::WAVE_BYTES, p.K, wave, lane, acc);
    // lane holds dot(W row n0 + b*16 + trow, X row j*16 + 4*kq + q) over its wavefront's share of K
    if (wave > 0) {
#pragma unroll
        for (int b = 0; b < SKINNY_BLKS; ++b)
#pragma unroll
            for (int j = 0; j < RB; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) red[wave - 1][b * 16 + trow][j * 16 + kq * 4 + q] = acc[b][j][q];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int b = 0; b < SKINNY_BLKS; ++b)
#pragma unroll
            for (int j = 0; j < RB; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = b * 16 + trow, t = j * 16 + kq * 4 + q;
                    red[0][c][t] = acc[b][j][q] + red[0][c][t] + red[1][c][t] + red[2][c][t];
                }
    }
    __syncthreads();
    // every thread finishes (row, column) pairs: column fastest, so a row's 32 outputs are one 64-byte store run
    for (int e = tid; e < T * SKINNY_ROWS; e += 256) {
        const int t = e / SKINNY_ROWS, c = e % SKINNY_ROWS, n = n0 + c;
        if (n < N) small_epilogue(p.epi, t, n, srow[t], red[0][c][t]);
    }
}

// ---- weight read N-contiguous (the input gradient through an nn.Linear weight, the forward through
// a Conv1D weight).  A workgroup owns COLGEMV_CT columns and one K range: it streams its
// [K range][CT] block of the weight once, 32 k-rows per step through LDS (three register sets: the
// rows of step s + 2 are requested while step s multiplies), reads the weight fragments with the
// transposing LDS load and the A fragments (at most 16 rows, from L2) straight from global memory,
// and leaves a [T][CT] fp32 partial sum per K range; symb_small_finish_kernel adds the ranges up in
// order and runs the epilogue.  grid = (ceil(N / CT), K ranges).
constexpr int COLGEMV_CT = 128;
struct ColGemvParams {
    const bf16* W;            // [K][N]
    const bf16* A;            // [T][K]
    float* partial;           // [ranges][16][N] fp32 (rows >= T never read back)
    int K, N, T;
    int k_per_range;          // a multiple of 32
};
__global__ void __launch_bounds__(256)
symb_colgemv_kernel(const ColGemvParams p) {
    constexpr int CT = COLGEMV_CT, NI = CT / 64, TT = 32;
    constexpr int RPITCH = CT * 2 + 16, LPRW = CT / 8, NRC = TT * LPRW / 256;
    __shared__ __attribute__((aligned(16))) unsigned char sW[TT * RPITCH];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c0 = blockIdx.x * CT;
    const int k_lo = blockIdx.y * p.k_per_range, k_hi = min(p.K, k_lo + p.k_per_range);
    floatx4 acc[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    struct Stage { u32x4 w[NRC]; u32x4 a; };
    const bool col_ok = (c0 + (tid % LPRW) * 8) < p.N;
    const int arow = lane & 15, akq = lane >> 4;         // this lane's A fragment: row arow, k = 8 akq .. + 7 of the step
    // every load is unconditional (clamped onto valid addresses) and zeroed when it is used: see symb_lora_grad_kernel
    auto fetch = [&](Stage& sg, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NRC; ++i) {
            const int c = tid + i * 256, kr = c / LPRW, cc = c % LPRW;
            sg.w[i] = ld_glb16(p.W + (size_t)min(k0 + kr, p.K - 1) * p.N + c0 + (col_ok ? cc * 8 : 0));
        }
        sg.a = ld_glb16(p.A + (size_t)min(arow, p.T - 1) * p.K + min(k0 + akq * 8, p.K - 8));
    };
    auto put = [&](const Stage& sg, int k0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NRC; ++i) {
            const int c = tid + i * 256, kr = c / LPRW, cc = c % LPRW;
            const bool ok = (k0 + kr) < k_hi && col_ok;
            *reinterpret_cast<u32x4*>(sW + kr * RPITCH + cc * 16) = ok ? sg.w[i] : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto multiply = [&](const Stage& sg, int k0) __attribute__((always_inline)) {
        const bool a_ok = arow < p.T && (k0 + akq * 8) < k_hi;          // K and the ranges are multiples of 8
        const bf16x8 af = __builtin_bit_cast(bf16x8, a_ok ? sg.a : u32x4{0u, 0u, 0u, 0u});
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bf16x8 wf = lds_read_tr_16x32(sW, RPITCH, wave * (NI * 16) + i * 16, lane);
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, af, acc[i], 0, 0, 0);
        }
    };
    if (k_lo < k_hi) {
        Stage sg0, sg1, sg2;
        fetch(sg0, k_lo);
        fetch(sg1, k_lo + TT);
        auto step = [&](Stage& cur, Stage& nxt, int k0) __attribute__((always_inline)) {
            __syncthreads();
            put(cur, k0);
            __syncthreads();
            fetch(nxt, k0 + 2 * TT);
            multiply(cur, k0);
        };
        for (int k0 = k_lo; k0 < k_hi; k0 += 3 * TT) {
            step(sg0, sg2, k0);
            if (k0 + TT < k_hi) step(sg1, sg0, k0 + TT);
            if (k0 + 2 * TT < k_hi) step(sg2, sg1, k0 + 2 * TT);
        }
    }
    // lane holds C[t = lane & 15][n = c0 + wave * NI * 16 + i * 16 + 4 (lane >> 4) + q]
    float* const out = p.partial + ((size_t)blockIdx.y * 16 + (lane & 15)) * p.N;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int n = c0 + wave * (NI * 16) + i * 16 + ((lane >> 4) << 2);
        if (n < p.N && (lane & 15) < p.T)
            *reinterpret_cast<float4*>(out + n) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    }
}

// Adds the K ranges of symb_colgemv_kernel up in order and finishes every (row, column) pair.
struct SmallFinishParams {
    const float* partial;     // [ranges][16][N]
    int ranges;
    SmallEpilogue epi;
};
__global__ void __launch_bounds__(256)
symb_small_finish_kernel(const SmallFinishParams p) {
    // grid = (column blocks of 256, rows): one (row, column) pair per thread, the ranges four at a time
    const int n = blockIdx.x * 256 + threadIdx.x, t = blockIdx.y;
    if (n >= p.epi.N) return;
    int s = 0;
    while (s + 1 < p.epi.S && t >= p.epi.off[s + 1]) ++s;
    const float* src = p.partial + (size_t)t * p.epi.N + n;
    const size_t stride = (size_t)16 * p.epi.N;
    float v = 0.f;
    int r = 0;
    for (; r + 4 <= p.ranges; r += 4) {
        const float a0 = src[(size_t)r * stride], a1 = src[(size_t)(r + 1) * stride], a2 = src[(size_t)(r + 2) * stride],
                    a3 = src[(size_t)(r + 3) * stride];
        v = (((v + a0) + a1) + a2) + a3;
    }
    for (; r < p.ranges; ++r) v += src[(size_t)r * stride];
    small_epilogue(p.epi, t, n, s, v);
}

// Packs B_i [d_out][r] into B_i^T [rpad][d_out] (zero rows beyond r) so the backward
// projection reads K-contiguous adapter rows.  grid.y = segment, grid.x covers d_out.
struct PackParams {
    const SegDesc* seg;
    bf16* packed;
    const int64_t* packed_off;
    int d_out;
};
__global__ void __launch_bounds__(256) symb_pack_bt_kernel(const PackParams p) {
    const SegDesc sd = p.seg[blockIdx.y];
    if (sd.kind != KIND_LORA) return;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= p.d_out) return;
    unsigned short* dst = reinterpret_cast<unsigned short*>(p.packed + p.packed_off[blockIdx.y]);
    const unsigned short* src = reinterpret_cast<const unsigned short*>(sd.B) + (size_t)j * sd.rank;
    for (int q = 0; q < sd.rpad; ++q) dst[(size_t)q * p.d_out + j] = (q < sd.rank) ? src[q] : (unsigned short)0;
}

// Packs A_i [r][d_in] into A_i^T [d_in][r] (exactly r columns): the adapter-side operand of the
// input gradient when the base weight is stored input-major (the K-contiguous GEMM then wants the
// adapter rows rank-contiguous per input column).  grid.y = segment, grid.x covers d_in.
struct PackAtParams {
    const SegDesc* seg;
    bf16* packed;
    const int64_t* packed_off;
    int d_in;
};
__global__ void __launch_bounds__(256) symb_pack_at_kernel(const PackAtParams p) {
    const SegDesc sd = p.seg[blockIdx.y];
    if (sd.kind != KIND_LORA) return;
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= p.d_in) return;
    unsigned short* dst = reinterpret_cast<unsigned short*>(p.packed + p.packed_off[blockIdx.y]) + (size_t)k * sd.rank;
    const unsigned short* src = reinterpret_cast<const unsigned short*>(sd.A);
    for (int q = 0; q < sd.rank; ++q) dst[q] = src[(size_t)q * p.d_in + k];
}

// -------------------------------------------------------------------------------------------
// LoRA parameter gradients of one segment, contraction over its tokens:
//   G[c][pp] = sum_t R[t][c] * L[t][pp]
//   dB_i (CMAJOR = true ): R = dY, L = Hs -> out[c * rank + pp]      ([d_out][r])
//   dA_i (CMAJOR = false): R = X,  L = dH -> out[pp * ncols + c]     ([r][d_in])
// A workgroup owns 256 columns (128 at ranks above 32) of one work item and walks its tokens 32 at a time through
// LDS; both MFMA operands are token-strided in memory and are read with the transposing
// LDS load.  A work item is a whole segment, or, for a segment of more than GRAD_SPLIT_MIN
// tokens, one of its runs of GRAD_SPLIT tokens: a long segment walked by one workgroup per
// column block would set the time of the whole launch.  Such a run leaves its sum in the
// workspace (same layout as the result) and symb_grad_reduce_kernel adds the runs up in
// order.  Fixed summation order, a function of the segment's length alone: results do not
// depend on the launch or on the rest of the batch.
// -------------------------------------------------------------------------------------------
constexpr int GRAD_SPLIT = 1024;       // tokens per run of a split segment (a multiple of GRAD_TT)
constexpr int GRAD_SPLIT_MIN = 1536;   // segments up to this length stay whole
struct GradItem {
    int32_t seg, t_lo, t_hi;  // tokens [t_lo, t_hi) of segment seg
    int32_t direct;           // 1: the result goes to the segment's dA / dB; 0: to partial + partial_off
    int64_t partial_off;      // in floats
};
struct GradParams {
    const bf16* R;            // [T][ncols]
    const bf16* L;            // [T][l_pitch]: per row rpad_i values then rpad_i residuals (see skinny kernel)
    int ncols, l_pitch;
    const int32_t* off;
    const SegDesc* seg;
    const GradItem* items;    // device: the work of this launch (grid.y indexes it)
    int accumulate;
    const bf16* const* R_seg; // device [S] or null: rows of segment i of R start at R_seg[i]
    float* partial;           // workspace region of the split segments' runs
};

template <int RB> constexpr int GRAD_CT = RB <= 2 ? 256 : 128;   // columns per workgroup (512-byte row pieces where the registers allow)
constexpr int GRAD_TT = 32;        // tokens per step

template <int RB, bool CMAJOR>
__global__ void __launch_bounds__(256)
symb_lora_grad_kernel(const GradParams p) {
    constexpr int CT = GRAD_CT<RB>, NI = CT / 64;           // columns per workgroup, 16-column blocks per wavefront
    constexpr int RPITCH = CT * 2 + 16;                    // LDS row pitch of the R tile in bytes
    constexpr int LPRW = CT / 8, NRC = GRAD_TT * LPRW / 256;   // 16-byte chunks per R row, R chunks per thread
    constexpr int LP = 2 * RB * 16 * 2 + 16;           // LDS row pitch of the L tile (value | residual) in bytes
    __shared__ __attribute__((aligned(16))) unsigned char sR[GRAD_TT * RPITCH];
    __shared__ __attribute__((aligned(16))) unsigned char sL[GRAD_TT * LP];
    const GradItem it = p.items[blockIdx.y];
    const int s = it.seg;
    const SegDesc sd = p.seg[s];
    const int t_lo = it.t_lo, t_hi = it.t_hi;
    const bf16* const rbase = p.R_seg ? p.R_seg[s] - (size_t)p.off[s] * p.ncols : p.R;
    const int c0 = blockIdx.x * CT;
    const int nb = sd.rpad >> 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    floatx4 acc[NI][RB];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < RB; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // R tile: 32 rows x CT/8 chunks of 8 columns, NRC per thread.  L tile: 32 x (rpad/4) chunks,
    // at most NLC per thread.  Two register sets: the chunks of tokens t0 + 64 are requested as soon as those
    // of t0 are in LDS (their set is free then), so a request has two steps to arrive (a step is far shorter than the memory
    // latency, and a launch over a few segments has too few workgroups per CU to hide it otherwise).
    // Every load is unconditional: out-of-range chunks read a valid address and count as zero when they go
    // to LDS, two steps later.  (With the zeroing next to the load the compiler puts the load under the
    // condition, and a load that may or may not have been issued makes it wait for all of them, the
    // newest request included.)
    constexpr int NLC = (GRAD_TT * 4 * RB + 255) / 256;
    const int lw = sd.rpad >> 2;                       // 16-byte chunks per L row: 2 * rpad bf16
    const int l_chunks = GRAD_TT * lw;
    struct Stage { u32x4 rr[NRC]; u32x4 lv[NLC]; };
    const bool col_ok = (c0 + (tid % LPRW) * 8) < p.ncols;
    auto fetch = [&](Stage& sg, int t0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NRC; ++i) {
            const int c = tid + i * 256, tr = c / LPRW, cc = c % LPRW;
            sg.rr[i] = ld_glb16(rbase + (size_t)min(t0 + tr, t_hi - 1) * p.ncols + c0 + (col_ok ? cc * 8 : 0));
        }
#pragma unroll
        for (int i = 0; i < NLC; ++i) {
            const int c = tid + i * 256, tr = c / lw, pc = c % lw;
            sg.lv[i] = ld_glb16(p.L + (size_t)min(t0 + tr, t_hi - 1) * p.l_pitch + pc * 8);
        }
    };
    // the chunks of tokens t0.., landed (see step), go to LDS
    auto put = [&](const Stage& sg, int t0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NRC; ++i) {
            const int c = tid + i * 256, tr = c / LPRW, cc = c % LPRW;
            const bool ok = (t0 + tr) < t_hi && col_ok;
            *reinterpret_cast<u32x4*>(sR + tr * RPITCH + cc * 16) = ok ? sg.rr[i] : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < NLC; ++i) {
            const int c = tid + i * 256, tr = c / lw, pc = c % lw;
            if (c < l_chunks) *reinterpret_cast<u32x4*>(sL + tr * LP + pc * 16) = (t0 + tr) < t_hi ? sg.lv[i] : u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto multiply = [&]() __attribute__((always_inline)) {
        bf16x8 rf[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) rf[i] = lds_read_tr_16x32(sR, RPITCH, wave * (NI * 16) + i * 16, lane);
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            if (j < nb) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {      // bf16 value, then its rounding residual
                    const bf16x8 lf = lds_read_tr_16x32(sL, LP, half * sd.rpad + j * 16, lane);
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        if constexpr (CMAJOR) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lf, rf[i], acc[i][j], 0, 0, 0);
                        else acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rf[i], lf, acc[i][j], 0, 0, 0);
                    }
                }
            }
        }
    };
    if (t_lo < t_hi) {
        Stage sg0, sg1;
        fetch(sg0, t_lo);
        fetch(sg1, t_lo + GRAD_TT);
        // Two register sets, two tiles in flight: a set is free again as soon as its tile is in LDS, so the
        // tile two steps ahead is requested into it; cur was requested two fetches ago, and the wait for it
        // leaves the newest fetch in flight.
        auto step = [&](Stage& cur, int t0) __attribute__((always_inline)) {
            __syncthreads();     // previous step's LDS reads are done
            put(cur, t0);
            __syncthreads();
            fetch(cur, t0 + 2 * GRAD_TT);
            multiply();
        };
        for (int t0 = t_lo; t0 < t_hi; t0 += 2 * GRAD_TT) {
            step(sg0, t0);
            if (t0 + GRAD_TT < t_hi) step(sg1, t0 + GRAD_TT);
        }
    }
    float* out = it.direct ? (CMAJOR ? sd.dB : sd.dA) : p.partial + it.partial_off;
    const bool accumulate = it.direct && p.accumulate;
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            if (j < nb) {
                if constexpr (CMAJOR) {
                    // lane: column c = .. + (lane & 15); registers: pp = j*16 + 4*(lane >> 4) + q
                    const int c = c0 + wave * (NI * 16) + i * 16 + (lane & 15);
                    if (c < p.ncols) {
                        const int pp0 = j * 16 + ((lane >> 4) << 2);
                        float* dst = out + (size_t)c * sd.rank + pp0;
                        float old[4] = {0.f, 0.f, 0.f, 0.f};        // all four read before the first store
                        if (accumulate) {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (pp0 + q < sd.rank) old[q] = dst[q];
                        }
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (pp0 + q < sd.rank) dst[q] = old[q] + acc[i][j][q];
                    }
                } else {
                    // lane: pp = j*16 + (lane & 15); registers: column c = .. + 4*(lane >> 4) + q
                    const int pp = j * 16 + (lane & 15);
                    const int c = c0 + wave * (NI * 16) + i * 16 + ((lane >> 4) << 2);
                    if (pp < sd.rank && c < p.ncols) {
                        float4* dst = reinterpret_cast<float4*>(out + (size_t)pp * p.ncols + c);
                        float4 v = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
                        if (accumulate) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
                        *dst = v;
                    }
                }
            }
        }
}

// -------------------------------------------------------------------------------------------
// dB_i and dH_i in ONE pass over dY (ranks up to 16).  Both products contract dY:
//   dB_i[c][pp] = sum_t dY[t][c] * Hs[t][pp]            (over the segment's tokens)
//   dH[t][pp]   = s_i * sum_c dY[t][c] * B_i[c][pp]     (over the output columns)
// and dY is by far the largest tensor either reads (T x d_out), so reading it once instead of
// twice saves its bytes.  A workgroup owns G column blocks of 256 columns of one work item
// (a segment, or a run of a long one) and walks its tokens 32 at a time; per step it visits its
// column blocks in turn: the dY tile goes through LDS as in symb_lora_grad_kernel and feeds
// (a) the dB accumulators of that block (transposing LDS reads, token-contracted) and (b) a
// 32 x 16 partial of dH over the block's columns (plain LDS reads, B_i^T fragments from the
// packed copy, held in registers).  After the last block of a step the four wavefronts' dH partials
// meet in LDS and the sum goes to dh_partial[group][t][16]; symb_dh_finish_kernel adds the
// groups in order, scales by s_i and writes dH as value + residual.  Fixed summation order
// everywhere: deterministic, no atomics.  dB comes out bit-identical to symb_lora_grad_kernel's.
// -------------------------------------------------------------------------------------------
struct DhDbParams {
    const bf16* R;            // dY [T][ncols]
    const bf16* L;            // Hs [T][l_pitch]: per row 16 values then 16 residuals
    const bf16* packed;       // B_i^T [16][ncols] per LoRA segment (symb_pack_bt_kernel), at packed_off[i]
    const int64_t* packed_off;
    int ncols, l_pitch;
    const int32_t* off;
    const SegDesc* seg;
    const GradItem* items;
    int accumulate;
    const bf16* const* R_seg;
    float* partial;           // dB runs of split segments
    float* dh_partial;        // [gridDim.x][T][16] fp32
    int T;
};

template <int I0, int I1, class F>
__device__ __forceinline__ void grad_static_for(F&& f) {
    if constexpr (I0 < I1) {
        f(std::integral_constant<int, I0>{});
        grad_static_for<I0 + 1, I1>(f);
    }
}

template <int G>
__global__ void __launch_bounds__(256)
symb_lora_dhdb_kernel(const DhDbParams p) {
    constexpr int CT = 256, NI = CT / 64;
    constexpr int RPITCH = CT * 2 + 16, LPRW = CT / 8, NRC = GRAD_TT * LPRW / 256;
    constexpr int LP = 2 * 16 * 2 + 16;
    __shared__ __attribute__((aligned(16))) unsigned char sR[GRAD_TT * RPITCH];
    __shared__ __attribute__((aligned(16))) unsigned char sL[GRAD_TT * LP];
    __shared__ __attribute__((aligned(16))) float red[4][GRAD_TT][16 + 4];
    const GradItem it = p.items[blockIdx.y];
    const int s = it.seg;
    const SegDesc sd = p.seg[s];
    const int t_lo = it.t_lo, t_hi = it.t_hi;
    const bf16* const rbase = p.R_seg ? p.R_seg[s] - (size_t)p.off[s] * p.ncols : p.R;
    const bf16* const bt = p.packed + p.packed_off[s];
    const int nblk = (p.ncols + CT - 1) / CT;
    const int cb0 = blockIdx.x * G, ncb = min(G, nblk - cb0);     // this workgroup's column blocks (uniform)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    floatx4 acc[G][NI];                                  // dB of every block of the group
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int i = 0; i < NI; ++i) acc[g][i] = floatx4{0.f, 0.f, 0.f, 0.f};
    // B_i^T fragments of this wavefront's 64 columns of every block: lane holds rank row lane & 15,
    // columns 8 (lane >> 4) .. + 7 of each of the two 32-column steps
    u32x4 btf[G][2];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int c = (cb0 + g) * CT + wave * 64 + ks * 32 + (lane >> 4) * 8;
            const bool ok = g < ncb && c < p.ncols;
            btf[g][ks] = ld_glb16(bt + (size_t)(lane & 15) * p.ncols + (ok ? c : 0));
            if (!ok) btf[g][ks] = u32x4{0u, 0u, 0u, 0u};
        }

    struct Stage { u32x4 rr[NRC]; u32x4 lv; };
    const int l_chunks = GRAD_TT * 4;                    // 16-byte chunks of the L tile: 32 rows x 64 bytes (16 values + 16 residuals)
    const int l_tr = (tid & 127) >> 2, l_pc = tid & 3;    // this thread's chunk of it
    // unconditional loads, zeroed on their way to LDS (see symb_lora_grad_kernel)
    auto fetch = [&](Stage& sg, int t0, int g) __attribute__((always_inline)) {
        const int c0 = (cb0 + min(g, ncb - 1)) * CT;
        const bool col_ok = (c0 + (tid % LPRW) * 8) < p.ncols;
#pragma unroll
        for (int i = 0; i < NRC; ++i) {
            const int c = tid + i * 256, tr = c / LPRW, cc = c % LPRW;
            sg.rr[i] = ld_glb16(rbase + (size_t)min(t0 + tr, t_hi - 1) * p.ncols + c0 + (col_ok ? cc * 8 : 0));
        }
        sg.lv = ld_glb16(p.L + (size_t)min(t0 + l_tr, t_hi - 1) * p.l_pitch + l_pc * 8);
    };
    auto put = [&](const Stage& sg, int t0, int g) __attribute__((always_inline)) {
        const int c0 = (cb0 + g) * CT;
        const bool col_ok = (c0 + (tid % LPRW) * 8) < p.ncols;
#pragma unroll
        for (int i = 0; i < NRC; ++i) {
            const int c = tid + i * 256, tr = c / LPRW, cc = c % LPRW;
            const bool ok = (t0 + tr) < t_hi && col_ok;
            *reinterpret_cast<u32x4*>(sR + tr * RPITCH + cc * 16) = ok ? sg.rr[i] : u32x4{0u, 0u, 0u, 0u};
        }
        if (g == 0 && tid < l_chunks)                    // the Hs rows of a step are the same for all its blocks
            *reinterpret_cast<u32x4*>(sL + l_tr * LP + l_pc * 16) = (t0 + l_tr) < t_hi ? sg.lv : u32x4{0u, 0u, 0u, 0u};
    };
    floatx4 dh[2];                                       // dH partial of the step: token blocks 0 / 1, this wavefront's columns
    auto multiply = [&](auto GC) __attribute__((always_inline)) {
        constexpr int g = decltype(GC)::value;
        bf16x8 rf[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) rf[i] = lds_read_tr_16x32(sR, RPITCH, wave * (NI * 16) + i * 16, lane);
#pragma unroll
        for (int half = 0; half < 2; ++half) {           // Hs value, then its rounding residual
            const bf16x8 lf = lds_read_tr_16x32(sL, LP, half * 16, lane);
#pragma unroll
            for (int i = 0; i < NI; ++i) acc[g][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lf, rf[i], acc[g][i], 0, 0, 0);
        }
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const u32x4 yv = *reinterpret_cast<const u32x4*>(sR + (tb * 16 + (lane & 15)) * RPITCH + (wave * 64 + ks * 32 + (lane >> 4) * 8) * 2);
                dh[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, btf[g][ks]), __builtin_bit_cast(bf16x8, yv), dh[tb], 0, 0, 0);
            }
    };
    // One tile = (token step, column block), blocks fastest.  Two register sets, the tile two ahead is
    // requested as soon as the current one is in LDS.
    auto advance = [&](int& t0, int& g) __attribute__((always_inline)) {
        if (++g == ncb) { g = 0; t0 += GRAD_TT; }
    };
    if (t_lo < t_hi) {
        Stage sg0, sg1;
        int ft = t_lo, fg = 0;                           // the next tile to request
        fetch(sg0, ft, fg); advance(ft, fg);
        fetch(sg1, ft, fg); advance(ft, fg);
        int t0 = t_lo, g = 0;                            // the tile being computed
        auto step = [&](Stage& cur) __attribute__((always_inline)) {
            if (g == 0) dh[0] = dh[1] = floatx4{0.f, 0.f, 0.f, 0.f};
            __syncthreads();                             // the previous tile's LDS reads are done
            put(cur, t0, g);
            __syncthreads();
            fetch(cur, ft, fg); advance(ft, fg);         // the set is free again: the tile two steps ahead goes into it
            // the block index selects registers: dispatch on it (uniform)
            grad_static_for<0, G>([&](auto GC) __attribute__((always_inline)) {
                if (g == decltype(GC)::value) multiply(GC);
            });
            if (g == ncb - 1) {
                // the step's dH partial over this workgroup's columns: wavefronts meet in LDS, fixed order
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    *reinterpret_cast<float4*>(&red[wave][tb * 16 + (lane & 15)][(lane >> 4) * 4]) = make_float4(dh[tb][0], dh[tb][1], dh[tb][2], dh[tb][3]);
                __syncthreads();
                if (tid < GRAD_TT * 4) {
                    const int tr = tid >> 2, q = (tid & 3) * 4;
                    if (t0 + tr < t_hi) {
                        float4 v = *reinterpret_cast<const float4*>(&red[0][tr][q]);
#pragma unroll
                        for (int w = 1; w < 4; ++w) {
                            const float4 a = *reinterpret_cast<const float4*>(&red[w][tr][q]);
                            v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
                        }
                        *reinterpret_cast<float4*>(p.dh_partial + ((size_t)blockIdx.x * p.T + t0 + tr) * 16 + q) = v;
                    }
                }
            }
            advance(t0, g);
        };
        while (t0 < t_hi) {
            step(sg0);
            if (t0 < t_hi) step(sg1);
        }
    }
    // ---- dB of every block, as symb_lora_grad_kernel<1, true> writes it
    float* out = it.direct ? sd.dB : p.partial + it.partial_off;
    const bool accumulate = it.direct && p.accumulate;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (g < ncb) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int c = (cb0 + g) * CT + wave * (NI * 16) + i * 16 + (lane & 15);
                if (c < p.ncols) {
                    const int pp0 = (lane >> 4) << 2;
                    float* dst = out + (size_t)c * sd.rank + pp0;
                    float old[4] = {0.f, 0.f, 0.f, 0.f};
                    if (accumulate) {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            if (pp0 + q < sd.rank) old[q] = dst[q];
                    }
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (pp0 + q < sd.rank) dst[q] = old[q] + acc[g][i][q];
                }
            }
        }
    }
}

// dH of the rows of one chunk from the groups' partial sums: dH[t][pp] = s_i * (group 0 + group 1 + ...),
// written as a bf16 value plus its bf16 rounding residual (the layout the skinny kernel writes).
struct DhFinishParams {
    const float* dh_partial;  // [groups][T][16]
    int groups, T;
    bf16* out;                // [T][out_pitch]
    int out_pitch;
    const RowChunk* chunks;
    const SegDesc* seg;
};
__global__ void __launch_bounds__(128)
symb_dh_finish_kernel(const DhFinishParams p) {
    const RowChunk ch = p.chunks[blockIdx.x];
    const SegDesc sd = p.seg[ch.seg];
    const int tr = threadIdx.x >> 2, q = (threadIdx.x & 3) * 4;
    if (tr >= ch.nrows) return;
    const size_t row = (size_t)(ch.row0 + tr);
    float4 v = *reinterpret_cast<const float4*>(p.dh_partial + row * 16 + q);
    for (int g = 1; g < p.groups; ++g) {
        const float4 a = *reinterpret_cast<const float4*>(p.dh_partial + ((size_t)g * p.T + row) * 16 + q);
        v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
    }
    v.x *= sd.scale; v.y *= sd.scale; v.z *= sd.scale; v.w *= sd.scale;
    const unsigned h01 = pack2_bf16(v.x, v.y), h23 = pack2_bf16(v.z, v.w);
    uint2 hi2, lo2;
    hi2.x = h01;
    hi2.y = h23;
    lo2.x = pack2_bf16(v.x - bf16_bits_to_f32((unsigned short)(h01 & 0xffffu)), v.y - bf16_bits_to_f32((unsigned short)(h01 >> 16)));
    lo2.y = pack2_bf16(v.z - bf16_bits_to_f32((unsigned short)(h23 & 0xffffu)), v.w - bf16_bits_to_f32((unsigned short)(h23 >> 16)));
    bf16* o = p.out + row * p.out_pitch;
    *reinterpret_cast<uint2*>(o + q) = hi2;
    *reinterpret_cast<uint2*>(o + sd.rpad + q) = lo2;
}

// Sums the runs of the split segments (see GradItem) into their dA / dB: element by element,
//   out = (accumulate ? out : 0) + (run 0 + run 1 + ...), the runs in this order.
// grid.y indexes the split segments; every thread owns four consecutive floats at a time.
struct GradReduceItem {
    int32_t seg, nruns;
    int64_t partial_off;      // run 0, in floats; run q follows at + q * rank * ncols
};
struct GradReduceParams {
    const SegDesc* seg;
    const GradReduceItem* items;
    const float* partial;
    int ncols, cmajor, accumulate;
};
__global__ void __launch_bounds__(256) symb_grad_reduce_kernel(const GradReduceParams p) {
    const GradReduceItem it = p.items[blockIdx.y];
    const SegDesc sd = p.seg[it.seg];
    const size_t n = (size_t)sd.rank * p.ncols;          // a multiple of 4: ncols is a multiple of 8
    float* const out = p.cmajor ? sd.dB : sd.dA;
    const float* const run0 = p.partial + it.partial_off;
    for (size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4; e < n; e += (size_t)gridDim.x * 1024) {
        float4 v = *reinterpret_cast<const float4*>(run0 + e);
        for (int q = 1; q < it.nruns; ++q) {
            const float4 a = *reinterpret_cast<const float4*>(run0 + (size_t)q * n + e);
            v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
        }
        if (p.accumulate) { const float4 o = *reinterpret_cast<const float4*>(out + e); v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
        *reinterpret_cast<float4*>(out + e) = v;
    }
}

// -------------------------------------------------------------------------------------------
// IA3 vector gradient:  dl_i[j] = sum_{t in segment i} dY[t][j] * Y0[t][j]
// grid.x covers d_out in blocks of 128 columns, grid.y indexes the IA3 segments that want it.
// A thread owns 8 columns (16-byte loads) and every 16th token, four tokens per step in flight;
// partial sums meet in LDS in a fixed order.
// -------------------------------------------------------------------------------------------
struct Ia3GradParams {
    const bf16* dY;
    const bf16* Y0;
    int d_out;
    const int32_t* off;
    const SegDesc* seg;
    const int32_t* seg_list;
    int accumulate;
    const bf16* const* dY_seg;   // device [S] or null: per-segment buffers of the first / second operand
    const bf16* const* Y0_seg;
};
constexpr int IA3_GRAD_COLS = 128;
__global__ void __launch_bounds__(256) symb_ia3_grad_kernel(const Ia3GradParams p) {
    __shared__ float red[16][16][9];
    const int s = p.seg_list[blockIdx.y];
    const int t_lo = p.off[s], t_hi = p.off[s + 1];
    const bf16* const gbase = p.dY_seg ? p.dY_seg[s] - (size_t)t_lo * p.d_out : p.dY;
    const bf16* const ybase = p.Y0_seg ? p.Y0_seg[s] - (size_t)t_lo * p.d_out : p.Y0;
    const int cc = threadIdx.x & 15, tl = threadIdx.x >> 4;
    const int c = blockIdx.x * IA3_GRAD_COLS + cc * 8;
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    auto fma8 = [&](const uint4& g, const uint4& y) __attribute__((always_inline)) {
        const unsigned int gw[4] = {g.x, g.y, g.z, g.w}, yw[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a[2 * q] += bf16_bits_to_f32((unsigned short)(gw[q] & 0xffffu)) * bf16_bits_to_f32((unsigned short)(yw[q] & 0xffffu));
            a[2 * q + 1] += bf16_bits_to_f32((unsigned short)(gw[q] >> 16)) * bf16_bits_to_f32((unsigned short)(yw[q] >> 16));
        }
    };
    if (c < p.d_out) {
        int t = t_lo + tl;
        for (; t + 48 < t_hi; t += 64) {
            uint4 g[4], y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                g[u] = *reinterpret_cast<const uint4*>(gbase + (size_t)(t + 16 * u) * p.d_out + c);
                y[u] = *reinterpret_cast<const uint4*>(ybase + (size_t)(t + 16 * u) * p.d_out + c);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) fma8(g[u], y[u]);
        }
        for (; t < t_hi; t += 16) {
            const uint4 g = *reinterpret_cast<const uint4*>(gbase + (size_t)t * p.d_out + c);
            const uint4 y = *reinterpret_cast<const uint4*>(ybase + (size_t)t * p.d_out + c);
            fma8(g, y);
        }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) red[tl][cc][q] = a[q];
    __syncthreads();
    if (tl == 0 && c < p.d_out) {
        float* out = p.seg[s].dA + c;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < 16; ++w) v += red[w][cc][q];
            out[q] = p.accumulate ? (out[q] + v) : v;
        }
    }
}

// -------------------------------------------------------------------------------------------
// Row scale for the IA3 backward:  out[t][j] = bf16( dY[t][j] * l_seg(t)[j] ) for IA3 rows,
// a plain copy for the others (and, with X and kind = IA3_IN, the input scale of the forward).  One workgroup per row chunk from the work list.
// -------------------------------------------------------------------------------------------
struct ScaleParams {
    const bf16* dY;           // [T][d_out]: rows to scale (dY for the IA3 backward, X for the IA3_IN forward)
    bf16* out;
    int d_out;                // row width
    const RowChunk* chunks;
    const SegDesc* seg;
    int kind;                 // segments of this kind are scaled by their vector, the others copied
    const bf16* const* in_seg;// device [S] or null: input rows of segment i start at in_seg[i]
    const int32_t* off;       // device [S+1] (read only with in_seg)
};
__global__ void __launch_bounds__(256) symb_ia3_scale_rows_kernel(const ScaleParams p) {
    const RowChunk ch = p.chunks[blockIdx.x];
    const SegDesc sd = p.seg[ch.seg];
    const bool ia3 = sd.kind == p.kind;
    const int nchunk = p.d_out >> 3;
    const bf16* const in = p.in_seg ? p.in_seg[ch.seg] - (size_t)p.off[ch.seg] * p.d_out : p.dY;
    // a thread keeps its 8 columns and walks the chunk's rows, four rows in flight
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        uint4 l = make_uint4(0u, 0u, 0u, 0u);
        if (ia3) l = *reinterpret_cast<const uint4*>(sd.A + c * 8);
        const unsigned int lw[4] = {l.x, l.y, l.z, l.w};
        auto scaled = [&](uint4 g) __attribute__((always_inline)) {
            if (ia3) {
                unsigned int gw[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float lo = bf16_bits_to_f32((unsigned short)(gw[q] & 0xffffu)) * bf16_bits_to_f32((unsigned short)(lw[q] & 0xffffu));
                    const float hi = bf16_bits_to_f32((unsigned short)(gw[q] >> 16)) * bf16_bits_to_f32((unsigned short)(lw[q] >> 16));
                    gw[q] = pack2_bf16(lo, hi);
                }
                g = make_uint4(gw[0], gw[1], gw[2], gw[3]);
            }
            return g;
        };
        const size_t col = (size_t)c * 8;
        int t = 0;
        for (; t + 4 <= ch.nrows; t += 4) {
            uint4 g[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) g[u] = *reinterpret_cast<const uint4*>(in + (size_t)(ch.row0 + t + u) * p.d_out + col);
#pragma unroll
            for (int u = 0; u < 4; ++u) *reinterpret_cast<uint4*>(p.out + (size_t)(ch.row0 + t + u) * p.d_out + col) = scaled(g[u]);
        }
        for (; t < ch.nrows; ++t) {
            const uint4 g = *reinterpret_cast<const uint4*>(in + (size_t)(ch.row0 + t) * p.d_out + col);
            *reinterpret_cast<uint4*>(p.out + (size_t)(ch.row0 + t) * p.d_out + col) = scaled(g);
        }
    }
}

// -------------------------------------------------------------------------------------------
// Noise prepass of the privacy flow:  out[t][k] = bf16( X[t][k] + n_seg(t)[r][k] ), r = 0 for a
// broadcast row, else the token's index inside its segment; rows of segments without noise are
// copied.  One workgroup per row chunk from the work list; fp32 sum, one rounding.
// -------------------------------------------------------------------------------------------
struct NoiseAddParams {
    const bf16* X;
    bf16* out;
    int width;
    const RowChunk* chunks;
    const int32_t* off;
    const NoiseDesc* noise;
};
__global__ void __launch_bounds__(256) symb_noise_add_kernel(const NoiseAddParams p) {
    const RowChunk ch = p.chunks[blockIdx.x];
    const NoiseDesc nd = p.noise[ch.seg];
    const int nchunk = p.width >> 3, seg0 = p.off[ch.seg];
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        const size_t col = (size_t)c * 8;
        for (int t = 0; t < ch.nrows; ++t) {
            const int row = ch.row0 + t;
            uint4 x = *reinterpret_cast<const uint4*>(p.X + (size_t)row * p.width + col);
            if (nd.ptr) {
                const uint4 n = *reinterpret_cast<const uint4*>(nd.ptr + (size_t)(nd.rows == 1 ? 0 : row - seg0) * p.width + col);
                unsigned int xw[4] = {x.x, x.y, x.z, x.w};
                const unsigned int nw[4] = {n.x, n.y, n.z, n.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float lo = bf16_bits_to_f32((unsigned short)(xw[q] & 0xffffu)) + bf16_bits_to_f32((unsigned short)(nw[q] & 0xffffu));
                    const float hi = bf16_bits_to_f32((unsigned short)(xw[q] >> 16)) + bf16_bits_to_f32((unsigned short)(nw[q] >> 16));
                    xw[q] = pack2_bf16(lo, hi);
                }
                x = make_uint4(xw[0], xw[1], xw[2], xw[3]);
            }
            *reinterpret_cast<uint4*>(p.out + (size_t)row * p.width + col) = x;
        }
    }
}

// -------------------------------------------------------------------------------------------
// Row scatter of a per-segment call whose output went through a flat copy in the workspace:
// row t of segment i moves from in[t] to out_seg[i][t - off[i]].  One workgroup per row chunk.
// -------------------------------------------------------------------------------------------
struct ScatterParams {
    const bf16* in;           // [T][width]
    int width;
    const RowChunk* chunks;
    bf16* const* out_seg;     // device [S]
    const int32_t* off;       // device [S+1]
};
__global__ void __launch_bounds__(256) symb_scatter_rows_kernel(const ScatterParams p) {
    const RowChunk ch = p.chunks[blockIdx.x];
    const int nchunk = p.width >> 3;
    bf16* const out = p.out_seg[ch.seg] - (size_t)p.off[ch.seg] * p.width;
    for (int e = threadIdx.x; e < ch.nrows * nchunk; e += 256) {
        const size_t at = (size_t)(ch.row0 + e / nchunk) * p.width + (size_t)(e % nchunk) * 8;
        *reinterpret_cast<uint4*>(out + at) = *reinterpret_cast<const uint4*>(p.in + at);
    }
}

__global__ void __launch_bounds__(256) symb_fill_zero_kernel(float* dst, size_t n) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = 0.f;
}

}  // namespace symb
