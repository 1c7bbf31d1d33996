// Host side of the C ABI declared in include/symb.h: argument checks, the segment
// planner, descriptor staging and the kernel launches.  Nothing here computes any part
// of the layer on the CPU; without a GPU every compute entry point fails with
// SYMB_ERR_DEVICE.
#include "../../include/symb.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <utility>
#include <vector>

#include "adapter_kernels.hpp"
#include "gemm16_kernel.hpp"

using namespace symb;

// Workspace of symb_base_linear_fwd_static: a file-scope array, so that entry point needs no device
// allocation at all.  In host code this name is only a stand-in for the symbol; the address
// of each device's copy is asked for once, in symb_create (hipGetSymbolAddress), and kept in the context.
static __device__ __align__(256) unsigned char symb_static_scratch[SYMB_STATIC_SCRATCH_BYTES];

// One workgroup per entry of `out`: the id of the XCD (hardware register XCC_ID) the workgroup runs on.
__global__ void symb_xcc_probe_kernel(int* out) {
    if (threadIdx.x == 0) {
        unsigned v;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
        out[blockIdx.x] = (int)(v & 0xfu);
    }
}

namespace {

thread_local std::string g_tls_error;

constexpr int kSlots = 32;                      // descriptor ring depth (a training step of 7 projections makes 21 different blobs)
constexpr size_t kSlotBytes = (size_t)2 << 20;  // capacity of one descriptor blob
constexpr int kSkinnyRows = SKINNY_ROWS;        // rows per skinny / scale work item
constexpr int kMaxTimed = 4096;                 // GEMM launches recorded between two timing reads
constexpr int kXccProbeGroups = 2048;           // workgroups of the XCD-rule measurement (8 rounds of 256)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int rpad_of(int r) { return (r + 15) / 16 * 16; }

}  // namespace

struct symb_context {
    int device = 0;
    unsigned char* host_ring = nullptr;   // pinned, kSlots * kSlotBytes
    unsigned char* dev_ring = nullptr;    // device, kSlots * kSlotBytes
    hipEvent_t slot_done[kSlots] = {};
    bool slot_used[kSlots] = {};
    int next_slot = 0;                    // the slot the next new blob goes to (round robin)
    int cur_slot = 0;                     // the slot this call's kernels read
    // what each slot's device copy holds: a call whose blob is already there (same bytes, copied on
    // the same stream) reads that copy instead of sending the bytes again
    size_t slot_size[kSlots] = {};
    uint64_t slot_hash[kSlots] = {};
    hipStream_t slot_stream[kSlots] = {};
    int64_t desc_sent = 0, desc_in_place = 0;
    int call_slot = -1;                   // the slot this call's descriptors went to (-1: none yet)
    std::string error;
    // measurement switches (symb_debug_set_option); all on by default
    bool opt_desc_reuse = true, opt_k_split = true, opt_small_rows = true, opt_skinny_deep = true;
    // Whether workgroup id mod 8 names the XCD a workgroup runs on, measured at creation: the K-split of
    // the GEMM keeps all parts of a tile on one XCD (behind one L2) and is used only if this holds.
    bool xcd_rule = false;
    int xcc_of_residue[8] = {-1, -1, -1, -1, -1, -1, -1, -1};
    unsigned char* static_scratch = nullptr;     // this device's copy of the file-scope scratch array
    std::vector<const void*> lds_attr_set;       // kernels whose dynamic-LDS limit was raised on this context's device
    // measurement hook: event pairs around GEMM launches
    bool timing = false;
    std::vector<hipEvent_t> tev;                 // 2 * kMaxTimed events, created on first enable
    struct Timed { int variant; double flops; };
    std::vector<Timed> timed;
};

namespace {

symb_status fail(symb_handle h, symb_status st, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (h) h->error = buf;
    g_tls_error = buf;
    return st;
}

#define SYMB_HIP(h, call)                                                                      \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(h, SYMB_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_));    \
    } while (0)

symb_status validate(symb_handle h, const symb_batch* b) {
    if (!b) return fail(h, SYMB_ERR_INVALID_ARG, "batch is null");
    if (b->d_in <= 0 || b->d_out <= 0) return fail(h, SYMB_ERR_INVALID_ARG, "d_in and d_out must be positive");
    if ((b->d_in % 8) || (b->d_out % 8)) return fail(h, SYMB_ERR_INVALID_ARG, "d_in and d_out must be multiples of 8");
    if (b->weight_layout != SYMB_WEIGHT_LINEAR && b->weight_layout != SYMB_WEIGHT_CONV1D)
        return fail(h, SYMB_ERR_INVALID_ARG, "unknown weight layout %d", b->weight_layout);
    if (b->num_segments < 0) return fail(h, SYMB_ERR_INVALID_ARG, "num_segments is negative");
    if (!b->seg_offsets) return fail(h, SYMB_ERR_INVALID_ARG, "seg_offsets is null");
    if (b->num_segments > 0 && !b->adapters) return fail(h, SYMB_ERR_INVALID_ARG, "adapters is null");
    if (b->seg_offsets[0] != 0) return fail(h, SYMB_ERR_BAD_SEGMENTS, "seg_offsets[0] must be 0");
    for (int i = 0; i < b->num_segments; ++i)
        if (b->seg_offsets[i + 1] < b->seg_offsets[i])
            return fail(h, SYMB_ERR_BAD_SEGMENTS, "seg_offsets decrease at segment %d", i);
    for (int i = 0; i < b->num_segments; ++i) {
        const symb_adapter& a = b->adapters[i];
        switch (a.kind) {
            case SYMB_ADAPTER_NONE: break;
            case SYMB_ADAPTER_LORA:
                if (a.rank < 1) return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: LoRA rank must be >= 1", i);
                if (a.rank > SYMB_MAX_RANK)
                    return fail(h, SYMB_ERR_UNSUPPORTED, "segment %d: LoRA rank %d exceeds SYMB_MAX_RANK", i, a.rank);
                if (!a.A || !a.B) return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: LoRA needs A and B", i);
                if (((uintptr_t)a.A & 15) || ((uintptr_t)a.dA & 15) || ((uintptr_t)a.dB & 3) || ((uintptr_t)a.B & 1))
                    return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: adapter pointer misaligned", i);
                if ((a.rank % 8) == 0 && ((uintptr_t)a.B & 15))
                    return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: B must be 16-byte aligned", i);
                break;
            case SYMB_ADAPTER_IA3:
                if (!a.A) return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: IA3 needs its vector in A", i);
                if (((uintptr_t)a.A & 15) || ((uintptr_t)a.dA & 15))
                    return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: adapter pointer misaligned", i);
                break;
            case SYMB_ADAPTER_IA3_IN:
                if (!a.A) return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: IA3 input scaling needs its vector in A", i);
                if (((uintptr_t)a.A & 15) || ((uintptr_t)a.dA & 15))
                    return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: adapter pointer misaligned", i);
                break;
            default: return fail(h, SYMB_ERR_INVALID_ARG, "segment %d: unknown adapter kind %d", i, a.kind);
        }
    }
    return SYMB_OK;
}

bool misaligned16(const void* p) { return ((uintptr_t)p & 15) != 0; }

// ---- planner (pure integer host work) ------------------------------------------------------
void plan_row_tiles(const symb_batch* b, int tile_m, std::vector<int32_t>& lo, std::vector<int32_t>& hi) {
    const int S = b->num_segments;
    const int32_t* off = b->seg_offsets;
    const int T = off[S];
    const int nt = (T + tile_m - 1) / tile_m;
    lo.assign(nt, 0);
    hi.assign(nt, -1);
    int s = 0;
    for (int u = 0; u < nt; ++u) {
        const int r0 = u * tile_m, r1 = std::min(T, r0 + tile_m);
        while (off[s + 1] <= r0) ++s;            // first segment that owns row r0 (non-empty by construction)
        int e = s;
        while (off[e + 1] < r1) ++e;             // segment that owns row r1 - 1
        lo[u] = s;
        hi[u] = e;
    }
}

// Per row tile: 1 if one of its segments is of `kind` (the tiles whose epilogue has rows to scale).
std::vector<int32_t> plan_tile_kind(const symb_batch* b, const std::vector<int32_t>& lo, const std::vector<int32_t>& hi, int kind) {
    std::vector<int32_t> v(lo.size(), 0);
    for (size_t u = 0; u < lo.size(); ++u)
        for (int i = lo[u]; i <= hi[u] && !v[u]; ++i) v[u] = b->adapters[i].kind == kind;
    return v;
}

// Row chunks of `rows` rows, never across a segment boundary; only_kind >= 0: of segments of that kind only.
void plan_chunks(const symb_batch* b, int rows, int only_kind, std::vector<RowChunk>& out) {
    out.clear();
    for (int i = 0; i < b->num_segments; ++i) {
        if (only_kind >= 0 && b->adapters[i].kind != only_kind) continue;
        for (int r = b->seg_offsets[i]; r < b->seg_offsets[i + 1]; r += rows)
            out.push_back(RowChunk{i, r, std::min(rows, b->seg_offsets[i + 1] - r), 0});
    }
}

struct BatchInfo {
    int S = 0, T = 0;
    int n_lora = 0, n_ia3 = 0, n_ia3in = 0;
    int max_rpad = 0;
    size_t packed_elems = 0;   // sum rpad_i * d_out over LoRA segments (packed B^T)
    size_t packed_at_elems = 0;// sum r_i * d_in over LoRA segments (packed A^T, input-major weight only)
};

BatchInfo inspect(const symb_batch* b) {
    BatchInfo bi;
    bi.S = b->num_segments;
    bi.T = b->seg_offsets[bi.S];
    for (int i = 0; i < bi.S; ++i) {
        const symb_adapter& a = b->adapters[i];
        if (a.kind == SYMB_ADAPTER_LORA) {
            ++bi.n_lora;
            bi.max_rpad = std::max(bi.max_rpad, rpad_of(a.rank));
            bi.packed_elems += (size_t)rpad_of(a.rank) * b->d_out;
            bi.packed_at_elems += align_up((size_t)a.rank * b->d_in, 8);
        } else if (a.kind == SYMB_ADAPTER_IA3) {
            ++bi.n_ia3;
        } else if (a.kind == SYMB_ADAPTER_IA3_IN) {
            ++bi.n_ia3in;
        }
    }
    return bi;
}

// Tile variants of the GEMM kernel (gemm16_kernel.hpp): 3 = 256x256 tile, taken when the problem has
// enough such tiles to fill the chip; 2 = 128x128 tile, for everything smaller.
int gemm_variant(int M, int N) {
    const long big = (long)((M + 255) / 256) * ((N + 255) / 256);
    return big >= 128 ? 3 : 2;
}
int gemm_tile_m(int M, int N) { return gemm_variant(M, N) == 3 ? 256 : 128; }

// Row tiles per group of the tile walk (a group is walked column by column, so the 32 tiles an XCD runs
// at once are g row tiles x 32 / g column tiles).  Measured on the Gemma2-27B-shaped launches (80 row
// tiles), GEMM calls of a step summed: g = 5 32.7 ms, 4 32.9, 6 33.1, 8 33.3, 10 33.1, 7 33.6, 16 34+:
// small groups win (most on the long-K shapes, 2-3 %), and a g that does not divide the row tiles loses
// (ragged last group, groups straddling the XCDs' runs).  That holds for launches of many rounds whose
// tiles cost the same.  Where row tiles differ (a mixed batch: a row tile of dozens of one-token LoRA
// segments takes far longer than one inside a long segment) small groups put more column tiles of the
// slowest row tile side by side and lose (+6 % on the mixed workload's step), and launches of two or
// three rounds do not care.  So: 8 unless the launch has at least five rounds per XCD and at most two
// segments per row tile; then the divisor of the row-tile count nearest 5 among 3..8, else 4.
int gemm_group_m(int num_m_tiles, int num_n_tiles, const std::vector<int32_t>& seg_lo, const std::vector<int32_t>& seg_hi) {
    int most = 0;
    for (size_t u = 0; u < seg_lo.size(); ++u) most = std::max(most, seg_hi[u] - seg_lo[u] + 1);
    if (most > 2 || ((long)num_m_tiles * num_n_tiles + 7) / 8 < 160) return 8;
    for (int g : {5, 4, 6, 3, 8, 7})
        if (num_m_tiles % g == 0) return g;
    return 4;
}

// K-split.  Every XCD walks a contiguous run of per_xcd = ceil(tiles / 8) tiles; the tiles of that run
// from number `whole` on are computed by `parts` workgroups each, one per K range, which leave fp32
// partial tiles in the workspace; the last one to arrive adds them up in part order and writes the
// tile.  Two uses:
//  * 128x128 tiles, launches that leave most of the chip idle (batches of a few hundred rows on a
//    4096-wide layer: 96 tiles for 256 CUs, each workgroup walking the whole K extent alone, a chain
//    of load and LDS latencies of about 0.5 us per 64 k): all tiles split (whole = 0),
//    parts = 320 / tiles: three parts for 96 tiles, none from 161 tiles on.
//  * 256x256 tiles, one workgroup per CU, 32 CUs per XCD: a run of per_xcd tiles ends in a round of
//    rem = per_xcd % 32 tiles that takes as long as a full one.  These last tiles are split into the
//    number of parts (at most 4) that makes the round shortest by a simple model of its time: e.g.
//    4 parts for 8 tiles (a quarter of a tile's time), 3 parts for 20 tiles of a long K (60
//    workgroups in two passes of a third each), none where the sum of the partial tiles (256 KiB
//    each) would cost what the split saves.
// parts is at most 8 and at most one per 8 stages of 64 k.  A pure function of the shape: the
// workspace figure does not depend on the process environment or on the handle.
struct SplitPlan {
    int parts = 1;        // K ranges per split tile (1: no split)
    int whole = 0;        // tiles per XCD that stay whole
    int slots = 0;        // split tiles of the launch (over all XCDs): arrival counters
    size_t bytes = 0;     // partial tiles: slots * parts * tile rows * tile columns * 4
};
SplitPlan gemm_split_plan(int M, int N, int K) {
    SplitPlan s;
    constexpr int target = 320, tail_max = 4;
    if (M <= 0) return s;
    const int KF = K / 64;
    if (gemm_variant(M, N) == 2) {
        const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
        const int P = std::min({8, KF / 8, (int)(target / tiles)});
        if (P < 2) return s;
        s.parts = P;
        s.slots = (int)tiles;                  // whole = 0: a tile's slot is its number in the walk
        s.bytes = (size_t)tiles * P * 128 * 128 * 4;
    } else {
        const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
        const int per_xcd = (int)((tiles + 7) / 8), rem = per_xcd % 32;
        if (rem == 0) return s;
        // The last round takes ceil(rem * P / 32) / P of a tile's time (a tile: about 1.45 us per stage)
        // plus, when split, about 8 + 4 P us for storing and adding up the partial tiles.
        const double tile_us = 1.45 * KF;
        int P = 1;
        double best = tile_us;
        for (int q = 2; q <= std::min(tail_max, KF / 8); ++q) {
            const double us = (double)((rem * q + 31) / 32) / q * tile_us + 8.0 + 4.0 * q;
            if (us < best - 4.0) { best = us; P = q; }      // a gain of a few us is not worth the traffic
        }
        if (P < 2 || best > 0.85 * tile_us) return s;      // nor is a gain of less than 15 % of the round
        s.parts = P;
        s.whole = per_xcd - rem;
        s.slots = 8 * rem;
        s.bytes = (size_t)s.slots * P * 256 * 256 * 4;
    }
    return s;
}

// One-pass dH + dB kernel: column blocks of 256 columns per workgroup (0: the layer is too narrow for it:
// with few column blocks the launch has too few workgroups, each walking its tokens alone, and the two
// separate passes are faster), and the number of workgroups along d_out.
int dhdb_blocks_per_group(int d_out) { return (d_out + 255) / 256 >= 64 ? 2 : 0; }
int dhdb_groups(int d_out) {
    const int g = dhdb_blocks_per_group(d_out);
    return g ? ((d_out + 255) / 256 + g - 1) / g : 0;
}

// LoRA gradients of long segments: a segment of more than GRAD_SPLIT_MIN tokens is walked in runs of
// GRAD_SPLIT tokens, each by workgroups of its own, which leave fp32 sums of the result's size in the
// workspace; a second kernel adds the runs up in order.  Number of runs of a segment of n tokens:
int grad_runs(int n) { return n > GRAD_SPLIT_MIN ? (n + GRAD_SPLIT - 1) / GRAD_SPLIT : 1; }
// Floats of workspace the runs of dB (of_b) or dA take for this batch.
size_t grad_split_floats(const symb_batch* b, bool of_b) {
    size_t n = 0;
    for (int i = 0; i < b->num_segments; ++i) {
        const symb_adapter& a = b->adapters[i];
        if (a.kind != SYMB_ADAPTER_LORA || !(of_b ? a.dB : a.dA)) continue;
        const int runs = grad_runs(b->seg_offsets[i + 1] - b->seg_offsets[i]);
        if (runs > 1) n += (size_t)runs * a.rank * (of_b ? b->d_out : b->d_in);
    }
    return n;
}

// Workspace layout (all regions 256-byte aligned, in this order; absent regions have size 0).
// Hs, dH and packed B^T sit at the same offsets for all three operations of one batch, so that a
// gradient call on the same workspace can take over what the forward call (Hs) and the
// input-gradient call (dH) left there (SYMB_GRAD_REUSE_HS / SYMB_GRAD_REUSE_DH).
struct WsLayout {
    size_t h_off = 0, h_bytes = 0;        // Hs  [T][2*max_rpad] bf16
    size_t dh_off = 0, dh_bytes = 0;      // dH  [T][2*max_rpad] bf16
    size_t pk_off = 0, pk_bytes = 0;      // packed B^T
    size_t sc_off = 0, sc_bytes = 0;      // IA3-scaled copy of dY [T][d_out] (input gradient) or of X [T][d_in] (forward, IA3_IN) bf16
    size_t pa_off = 0, pa_bytes = 0;      // packed A^T (input-major weight, input gradient only)
    size_t so_off = 0, so_bytes = 0;      // flat output [T][width] bf16 of a per-segment call whose outputs overlap its inputs
    size_t gr_off = 0, gr_bytes = 0;      // fp32 runs of the LoRA gradients of split segments (see grad_split)
    size_t dp_off = 0, dp_bytes = 0;      // fp32 partial sums of dH per group of column blocks (one-pass dH + dB, ranks up to 16)
    // optional regions (a workspace that ends before them makes the call take the tiled kernel, unsplit):
    size_t sg_off = 0, sg_bytes = 0;      // calls of at most 16 rows: flat copy of the activation rows [T][K] (gathered / scaled)
    size_t sp_off = 0, sp_bytes = 0;      // calls of at most 16 rows, weight read N-contiguous: fp32 partial sums per K range
    size_t tp_off = 0, tp_bytes = 0;      // fp32 partial tiles of a K-split GEMM (see gemm_split_plan); last
    size_t mandatory = 0;                 // end of the regions a call cannot do without
    size_t total = 0;
};

// K ranges of the small-batch kernel that reads the weight N-contiguous: enough workgroups to fill the
// chip (about 512 with the column blocks), at least 128 k per range, at most 8 MiB of partial sums
// (they are written and read back once: traffic beside the weight's own bytes).
constexpr int kSmallRows = 16;
int small_k_ranges(int K, int N) {
    const int nblk = (N + COLGEMV_CT - 1) / COLGEMV_CT;
    const long cap = std::max<long>(1, ((long)8 << 20) / ((long)kSmallRows * N * 4));
    return (int)std::max<long>(1, std::min<long>({(512 + nblk - 1) / nblk, (long)K / 128, cap}));
}
int small_k_per_range(int K, int N) {
    const int r = small_k_ranges(K, N);
    return (int)align_up((size_t)(K + r - 1) / r, 32);
}

WsLayout ws_layout(const symb_batch* b, const BatchInfo& bi, int op, bool full_bwd, bool any_lora_grad, bool staged_out = false) {
    WsLayout w;
    size_t cur = 0;
    auto take = [&](size_t& off, size_t& bytes, size_t n) {
        off = cur;
        bytes = n;
        cur += align_up(n, 256);
    };
    const size_t hb = (size_t)bi.T * (2 * bi.max_rpad) * 2;   // value + residual halves
    const bool conv1d = b->weight_layout == SYMB_WEIGHT_CONV1D;
    if (op == SYMB_OP_FWD) {
        if (bi.n_lora) take(w.h_off, w.h_bytes, hb);
        if (bi.n_lora && conv1d) {            // the N-contiguous GEMM wants B_i^T: same packing as the input gradient's
            take(w.dh_off, w.dh_bytes, hb);   // (gap: keeps packed B^T where the other operations have it)
            take(w.pk_off, w.pk_bytes, bi.packed_elems * 2);
        }
        if (bi.n_ia3in) take(w.sc_off, w.sc_bytes, (size_t)bi.T * b->d_in * 2);   // X with IA3_IN rows scaled
    } else if (op == SYMB_OP_BWD_INPUT) {
        if (full_bwd && bi.n_lora) {
            take(w.h_off, w.h_bytes, hb);     // not touched here: keeps the forward call's Hs intact
            take(w.dh_off, w.dh_bytes, hb);
            take(w.pk_off, w.pk_bytes, bi.packed_elems * 2);
        }
        if (full_bwd && bi.n_ia3) take(w.sc_off, w.sc_bytes, (size_t)bi.T * b->d_out * 2);
        if (full_bwd && bi.n_lora && conv1d) take(w.pa_off, w.pa_bytes, bi.packed_at_elems * 2);
    } else {
        if (any_lora_grad) {
            take(w.h_off, w.h_bytes, hb);
            take(w.dh_off, w.dh_bytes, hb);
            take(w.pk_off, w.pk_bytes, bi.packed_elems * 2);
            const size_t gr = std::max(grad_split_floats(b, true), grad_split_floats(b, false)) * 4;   // dB's runs, then dA's, in the same place
            if (gr) take(w.gr_off, w.gr_bytes, gr);
            if (bi.max_rpad == 16 && dhdb_groups(b->d_out)) take(w.dp_off, w.dp_bytes, (size_t)dhdb_groups(b->d_out) * bi.T * 16 * 4);
        }
    }
    if (staged_out && op != SYMB_OP_ADAPTER_GRAD)
        take(w.so_off, w.so_bytes, (size_t)bi.T * (op == SYMB_OP_FWD ? b->d_out : b->d_in) * 2);
    w.mandatory = cur;
    if (op != SYMB_OP_ADAPTER_GRAD && bi.T > 0 && bi.T <= kSmallRows) {
        // the contraction runs over d_in in the forward, over d_out in the input gradient; the weight is
        // read N-contiguous by the forward of an input-major weight and by the input gradient of an nn.Linear one
        const int K = op == SYMB_OP_FWD ? b->d_in : b->d_out, N = op == SYMB_OP_FWD ? b->d_out : b->d_in;
        take(w.sg_off, w.sg_bytes, (size_t)bi.T * K * 2);
        if ((op == SYMB_OP_FWD) == conv1d) {
            const int kpr = small_k_per_range(K, N);
            take(w.sp_off, w.sp_bytes, (size_t)((K + kpr - 1) / kpr) * kSmallRows * N * 4);
        }
    }
    if (op == SYMB_OP_FWD) {
        const SplitPlan sp = gemm_split_plan(bi.T, b->d_out, b->d_in);
        if (sp.parts > 1) take(w.tp_off, w.tp_bytes, sp.bytes);
    } else if (op == SYMB_OP_BWD_INPUT) {
        const SplitPlan sp = gemm_split_plan(bi.T, b->d_in, b->d_out);
        if (sp.parts > 1) take(w.tp_off, w.tp_bytes, sp.bytes);
    }
    w.total = cur;
    return w;
}

// ---- descriptor blob -------------------------------------------------------------------------
struct Blob {
    std::vector<unsigned char> bytes;
    template <class T>
    size_t add(const T* p, size_t n) {
        const size_t off = align_up(bytes.size(), 16);
        bytes.resize(off + std::max<size_t>(n, 1) * sizeof(T));
        if (n) memcpy(bytes.data() + off, p, n * sizeof(T));
        return off;
    }
};

symb_status upload(symb_handle h, const Blob& blob, hipStream_t st, unsigned char** dev_base) {
    if (blob.bytes.size() > kSlotBytes)
        return fail(h, SYMB_ERR_UNSUPPORTED, "batch descriptors need %zu bytes, capacity is %zu", blob.bytes.size(), kSlotBytes);
    // The kernels only read a slot's device copy (the K-split arrival counters are back at zero when
    // a launch ends), so a batch that comes again with the same offsets, adapters and buffers -- the
    // next decode step of the same clients, the same projection in the next training step -- finds
    // its descriptors in place.  The pinned copy of a slot is what its device copy holds.
    const bool reuse = h->opt_desc_reuse;
    const size_t n = blob.bytes.size();
    uint64_t hash = 0x9E3779B97F4A7C15ull ^ n;
    {
        size_t i = 0;
        for (; i + 8 <= n; i += 8) {
            uint64_t w;
            memcpy(&w, blob.bytes.data() + i, 8);
            hash = (hash ^ w) * 0x100000001B3ull;
            hash ^= hash >> 29;
        }
        for (; i < n; ++i) hash = (hash ^ blob.bytes[i]) * 0x100000001B3ull;
    }
    if (reuse)
        for (int j = 0; j < kSlots; ++j)
            if (h->slot_used[j] && h->slot_size[j] == n && h->slot_hash[j] == hash && h->slot_stream[j] == st &&
                memcmp(h->host_ring + (size_t)j * kSlotBytes, blob.bytes.data(), n) == 0) {
                h->cur_slot = j;
                h->call_slot = j;
                ++h->desc_in_place;
                *dev_base = h->dev_ring + (size_t)j * kSlotBytes;
                return SYMB_OK;
            }
    const int slot = h->next_slot;
    h->next_slot = (slot + 1) % kSlots;
    h->cur_slot = slot;
    h->call_slot = slot;
    if (h->slot_used[slot]) SYMB_HIP(h, hipEventSynchronize(h->slot_done[slot]));
    h->slot_used[slot] = false;            // until the copy is enqueued, the slot holds nothing a later call may reuse
    unsigned char* hp = h->host_ring + (size_t)slot * kSlotBytes;
    unsigned char* dp = h->dev_ring + (size_t)slot * kSlotBytes;
    memcpy(hp, blob.bytes.data(), n);
    SYMB_HIP(h, hipMemcpyAsync(dp, hp, n, hipMemcpyHostToDevice, st));
    ++h->desc_sent;
    h->slot_size[slot] = n;
    h->slot_hash[slot] = hash;
    h->slot_stream[slot] = st;
    h->slot_used[slot] = true;
    SYMB_HIP(h, hipEventRecord(h->slot_done[slot], st));   // a call that fails before its kernels still leaves the slot guarded
    *dev_base = dp;
    return SYMB_OK;
}

// A call that fails after its descriptors went to a slot may leave that slot's device copy in a state
// no later call should take over (a GEMM that never ran has not put its K-split counters back to zero, a
// launch may be half enqueued): unless the call completes, its slot is never matched again.
struct CallGuard {
    symb_handle h;
    bool completed = false;
    explicit CallGuard(symb_handle h_) : h(h_) { h->call_slot = -1; }
    ~CallGuard() {
        if (!completed && h->call_slot >= 0) h->slot_size[h->call_slot] = SIZE_MAX;
    }
};

// Marks the slot busy until everything enqueued so far on `st` has run (kernels read it).
symb_status seal_slot(symb_handle h, hipStream_t st) {
    SYMB_HIP(h, hipEventRecord(h->slot_done[h->cur_slot], st));
    return SYMB_OK;
}

std::vector<SegDesc> make_segdesc(const symb_batch* b) {
    std::vector<SegDesc> v(b->num_segments);
    for (int i = 0; i < b->num_segments; ++i) {
        const symb_adapter& a = b->adapters[i];
        SegDesc d{};
        d.kind = a.kind;
        d.rank = a.kind == SYMB_ADAPTER_LORA ? a.rank : 0;
        d.rpad = rpad_of(d.rank);
        d.scale = a.kind == SYMB_ADAPTER_LORA ? a.scale : 0.f;
        d.A = (const bf16*)a.A;
        d.B = (const bf16*)a.B;
        d.dA = (float*)a.dA;
        d.dB = (float*)a.dB;
        v[i] = d;
    }
    return v;
}

// ---- GEMM launch -----------------------------------------------------------------------------
template <class KFN>
symb_status launch_gemm_fn(symb_handle h, GemmParams gp, hipStream_t st, KFN kfn, int BM, int BN, int threads, int smem, int variant) {
    // once per context (= per device): the attribute belongs to the device the kernel is loaded on
    const void* kptr = reinterpret_cast<const void*>(kfn);
    if (std::find(h->lds_attr_set.begin(), h->lds_attr_set.end(), kptr) == h->lds_attr_set.end()) {
        SYMB_HIP(h, hipFuncSetAttribute(kptr, hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        h->lds_attr_set.push_back(kptr);
    }
    gp.num_m_tiles = (gp.M + BM - 1) / BM;
    gp.num_n_tiles = (gp.N + BN - 1) / BN;
    if (gp.group_m <= 0) gp.group_m = 8;
    const int total = gp.num_m_tiles * gp.num_n_tiles;
    const int per_xcd = (total + 7) / 8;
    int grid = per_xcd * 8;
    if (gp.k_parts > 1) grid = 8 * (gp.k_whole + (per_xcd - gp.k_whole) * gp.k_parts);
    const bool timed = h->timing && (int)h->timed.size() < kMaxTimed;
    const size_t slot = h->timed.size();
    if (timed) SYMB_HIP(h, hipEventRecord(h->tev[2 * slot], st));
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(threads), smem, st, gp);
    SYMB_HIP(h, hipGetLastError());
    if (timed) {
        SYMB_HIP(h, hipEventRecord(h->tev[2 * slot + 1], st));
        h->timed.push_back({variant, gp.timing_flops});
    }
    return SYMB_OK;
}

template <int NBLK, bool NN, bool PLAIN>
symb_status launch_gemm16_t(symb_handle h, const GemmParams& gp, hipStream_t st) {
    using TT = Gemm16Tile<NBLK>;
    // instantiation number of the measurement hook: bit 0 = N-contiguous weight, bit 1 = 128x128 tile, bit 2 = full epilogue
    constexpr int variant = (NN ? 1 : 0) | (NBLK == 4 ? 2 : 0) | (PLAIN ? 0 : 4);
    return launch_gemm_fn(h, gp, st, symb_gemm16_kernel<NBLK, NN, PLAIN>, TT::BM, TT::BN, TT::NT, TT::SMEM, variant);
}

// Algorithmic work of one GEMM launch: 2 M N K plus the fused LoRA term.
double gemm_flops(const symb_batch* b, int N, int K, bool lora) {
    const int S = b->num_segments;
    double f = 2.0 * b->seg_offsets[S] * (double)N * K;
    if (lora)
        for (int i = 0; i < S; ++i)
            if (b->adapters[i].kind == SYMB_ADAPTER_LORA)
                f += 2.0 * (b->seg_offsets[i + 1] - b->seg_offsets[i]) * (double)b->adapters[i].rank * N;
    return f;
}

template <bool NN>
symb_status launch_gemm(symb_handle h, const GemmParams& gp, hipStream_t st) {
    const bool plain = !gp.bias && !gp.epi_ia3 && !gp.Cbase && !gp.neff;
    if (gemm_variant(gp.M, gp.N) == 3) return plain ? launch_gemm16_t<8, NN, true>(h, gp, st) : launch_gemm16_t<8, NN, false>(h, gp, st);
    return plain ? launch_gemm16_t<4, NN, true>(h, gp, st) : launch_gemm16_t<4, NN, false>(h, gp, st);
}

// Up to one workgroup per compute unit the deep-prefetch build is used (where its buffers fit in LDS).
template <int RB>
void launch_skinny_rb(const SkinnyParams& sp, int nchunks, bool deep_ok, hipStream_t st) {
    if constexpr (RB <= 4) {
        if (deep_ok && nchunks <= 256) {
            hipLaunchKernelGGL((symb_skinny_kernel<RB, true>), dim3(nchunks), dim3(256), 0, st, sp);
            return;
        }
    }
    hipLaunchKernelGGL((symb_skinny_kernel<RB, false>), dim3(nchunks), dim3(256), 0, st, sp);
}
symb_status launch_skinny(symb_handle h, const SkinnyParams& sp, int nchunks, int max_rpad, hipStream_t st) {
    if (nchunks == 0) return SYMB_OK;
    const bool deep = h->opt_skinny_deep;
    if (max_rpad <= 16) launch_skinny_rb<1>(sp, nchunks, deep, st);
    else if (max_rpad <= 32) launch_skinny_rb<2>(sp, nchunks, deep, st);
    else if (max_rpad <= 64) launch_skinny_rb<4>(sp, nchunks, deep, st);
    else launch_skinny_rb<8>(sp, nchunks, deep, st);
    SYMB_HIP(h, hipGetLastError());
    return SYMB_OK;
}

template <int RB, bool CM>
void launch_grad_rb(const GradParams& gp, int nitems, hipStream_t st) {
    hipLaunchKernelGGL((symb_lora_grad_kernel<RB, CM>), dim3((gp.ncols + GRAD_CT<RB> - 1) / GRAD_CT<RB>, nitems), dim3(256), 0, st, gp);
}
template <bool CM>
symb_status launch_grad(symb_handle h, const GradParams& gp, int nseg, int max_rpad, hipStream_t st) {
    if (nseg == 0) return SYMB_OK;
    if (max_rpad <= 16) launch_grad_rb<1, CM>(gp, nseg, st);
    else if (max_rpad <= 32) launch_grad_rb<2, CM>(gp, nseg, st);
    else if (max_rpad <= 64) launch_grad_rb<4, CM>(gp, nseg, st);
    else launch_grad_rb<8, CM>(gp, nseg, st);
    SYMB_HIP(h, hipGetLastError());
    return SYMB_OK;
}
// Adds up the runs of the split segments (none: nothing to do).  At most 128 * 36864 floats per segment
// at 1024 per workgroup and pass.
symb_status launch_grad_reduce(symb_handle h, const GradReduceParams& rp, int nsplit, hipStream_t st) {
    if (nsplit == 0) return SYMB_OK;
    hipLaunchKernelGGL(symb_grad_reduce_kernel, dim3(1024, nsplit), dim3(256), 0, st, rp);
    SYMB_HIP(h, hipGetLastError());
    return SYMB_OK;
}

// C[T][N] = A[T][K] Wop, T <= 16, with the weight-streaming kernels (adapter_kernels.hpp).
//   w_kmajor: Wop is [N][K] (one workgroup per 32 columns, K split inside the workgroup);
//   else Wop is [K][N] (column blocks x K ranges, fp32 partial sums in `partial`, then the finish kernel).
symb_status launch_small(symb_handle h, const bf16* A, const bf16* Wop, bool w_kmajor, int K, const SmallEpilogue& epi,
                         float* partial, hipStream_t st) {
    if (w_kmajor) {
        RowGemvParams rp{Wop, A, K, epi};
        hipLaunchKernelGGL(symb_rowgemv_kernel<1>, dim3((epi.N + SKINNY_ROWS - 1) / SKINNY_ROWS), dim3(256), 0, st, rp);
        SYMB_HIP(h, hipGetLastError());
        return SYMB_OK;
    }
    const int kpr = small_k_per_range(K, epi.N), ranges = (K + kpr - 1) / kpr;
    ColGemvParams cp{Wop, A, partial, K, epi.N, epi.T, kpr};
    hipLaunchKernelGGL(symb_colgemv_kernel, dim3((epi.N + COLGEMV_CT - 1) / COLGEMV_CT, ranges), dim3(256), 0, st, cp);
    SYMB_HIP(h, hipGetLastError());
    SmallFinishParams fp{partial, ranges, epi};
    hipLaunchKernelGGL(symb_small_finish_kernel, dim3((epi.N + 255) / 256, epi.T), dim3(256), 0, st, fp);
    SYMB_HIP(h, hipGetLastError());
    return SYMB_OK;
}

// Whether a call of T rows takes the small-batch kernels: a handful of rows, the optional workspace
// regions present, and, for a weight read K-contiguous, a layer of moderate size (one workgroup per 32
// columns holds 152 KiB of LDS: on 4096 x 11008 the 344 workgroups make a second, third-full round and
// the tiled kernel with its K-split is faster at any row count).
bool small_path(symb_handle h, int T, bool w_kmajor, long long weights, bool second_output, const WsLayout& wl, const void* ws,
                size_t ws_bytes) {
    if (!h->opt_small_rows || T > kSmallRows || !wl.sg_bytes || !ws) return false;
    if (ws_bytes < (wl.sp_bytes ? wl.sp_off + wl.sp_bytes : wl.sg_off + wl.sg_bytes)) return false;
    // (a call with a pre-adapter output cannot split K in the tiled kernel: there the streaming kernel wins on any layer)
    return !w_kmajor || weights <= 24ll << 20 || second_output;
}

symb_status check_handle(symb_handle h) {
    if (!h) return fail(nullptr, SYMB_ERR_INVALID_ARG, "handle is null");
    if (hipSetDevice(h->device) != hipSuccess) return fail(h, SYMB_ERR_DEVICE, "hipSetDevice(%d) failed", h->device);
    return SYMB_OK;
}

}  // namespace

// =============================================================================================
extern "C" {

const char* symb_status_string(symb_status s) {
    switch (s) {
        case SYMB_OK: return "SYMB_OK";
        case SYMB_ERR_INVALID_ARG: return "SYMB_ERR_INVALID_ARG";
        case SYMB_ERR_BAD_SEGMENTS: return "SYMB_ERR_BAD_SEGMENTS";
        case SYMB_ERR_UNSUPPORTED: return "SYMB_ERR_UNSUPPORTED";
        case SYMB_ERR_WORKSPACE_TOO_SMALL: return "SYMB_ERR_WORKSPACE_TOO_SMALL";
        case SYMB_ERR_DEVICE: return "SYMB_ERR_DEVICE";
    }
    return "SYMB_ERR_UNKNOWN";
}

const char* symb_last_error(symb_handle h) { return h ? h->error.c_str() : g_tls_error.c_str(); }

symb_status symb_create(symb_handle* out, int device) {
    if (!out) return fail(nullptr, SYMB_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return fail(nullptr, SYMB_ERR_DEVICE, "no HIP device available");
    if (device < 0 || device >= ndev) return fail(nullptr, SYMB_ERR_INVALID_ARG, "device %d out of range (%d devices)", device, ndev);
    SYMB_HIP(nullptr, hipSetDevice(device));
    symb_context* c = new symb_context();
    c->device = device;
    if (hipHostMalloc((void**)&c->host_ring, kSlots * kSlotBytes, hipHostMallocDefault) != hipSuccess ||
        hipMalloc((void**)&c->dev_ring, kSlots * kSlotBytes) != hipSuccess) {
        if (c->host_ring) (void)hipHostFree(c->host_ring);
        delete c;
        return fail(nullptr, SYMB_ERR_DEVICE, "descriptor staging allocation failed");
    }
    for (int i = 0; i < kSlots; ++i) {
        if (hipEventCreateWithFlags(&c->slot_done[i], hipEventDisableTiming) != hipSuccess) {
            delete c;
            return fail(nullptr, SYMB_ERR_DEVICE, "hipEventCreate failed");
        }
    }
    // The K-split of the GEMM assumes that workgroup id mod 8 names the XCD: measure it.  Every
    // workgroup of a probe launch records the XCD it ran on; the rule holds if all workgroups of a
    // residue class report the same one.  (A device with a single XCD passes trivially.)
    {
        int* probe = reinterpret_cast<int*>(c->dev_ring);          // the ring is idle: borrow its first 8 KiB
        std::vector<int> xcc(kXccProbeGroups, -1);
        hipLaunchKernelGGL(symb_xcc_probe_kernel, dim3(kXccProbeGroups), dim3(64), 0, nullptr, probe);
        if (hipGetLastError() != hipSuccess ||
            hipMemcpy(xcc.data(), probe, sizeof(int) * kXccProbeGroups, hipMemcpyDeviceToHost) != hipSuccess) {
            symb_destroy(c);
            return fail(nullptr, SYMB_ERR_DEVICE, "XCD probe launch failed");
        }
        bool ok = true;
        for (int i = 0; i < kXccProbeGroups; ++i) ok = ok && xcc[i] == xcc[i & 7];
        c->xcd_rule = ok;
        for (int r = 0; r < 8; ++r) c->xcc_of_residue[r] = xcc[r];
    }
    {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(symb_static_scratch)) != hipSuccess || !p) {
            symb_destroy(c);
            return fail(nullptr, SYMB_ERR_DEVICE, "hipGetSymbolAddress(symb_static_scratch) failed");
        }
        c->static_scratch = static_cast<unsigned char*>(p);
    }
    *out = c;
    return SYMB_OK;
}

symb_status symb_debug_set_option(symb_handle h, int32_t option, int32_t value) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    switch (option) {
        case SYMB_OPT_DESCRIPTOR_REUSE: h->opt_desc_reuse = value != 0; break;
        case SYMB_OPT_K_SPLIT: h->opt_k_split = value != 0; break;
        case SYMB_OPT_SMALL_BATCH_KERNELS: h->opt_small_rows = value != 0; break;
        case SYMB_OPT_SKINNY_DEEP: h->opt_skinny_deep = value != 0; break;
        default: return fail(h, SYMB_ERR_INVALID_ARG, "unknown option %d", option);
    }
    return SYMB_OK;
}

symb_status symb_debug_xcd_rule(symb_handle h, int32_t* holds, int32_t* xcc_of_residue) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (holds) *holds = h->xcd_rule ? 1 : 0;
    if (xcc_of_residue)
        for (int r = 0; r < 8; ++r) xcc_of_residue[r] = h->xcc_of_residue[r];
    return SYMB_OK;
}

symb_status symb_debug_descriptor_stats(symb_handle h, int64_t* sent, int64_t* in_place) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (sent) *sent = h->desc_sent;
    if (in_place) *in_place = h->desc_in_place;
    return SYMB_OK;
}

symb_status symb_debug_gemm_timing_enable(symb_handle h, int32_t on) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (on && h->tev.empty()) {
        h->tev.resize(2 * kMaxTimed);
        for (auto& e : h->tev) SYMB_HIP(h, hipEventCreate(&e));
        h->timed.reserve(kMaxTimed);
    }
    h->timing = on != 0;
    h->timed.clear();
    return SYMB_OK;
}

symb_status symb_debug_gemm_timing_read(symb_handle h, int32_t variant, double* ms_total, int64_t* launches,
                                        double* flops_total) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (!ms_total || !launches || !flops_total) return fail(h, SYMB_ERR_INVALID_ARG, "null output pointer");
    *ms_total = 0.0;
    *launches = 0;
    *flops_total = 0.0;
    for (size_t i = 0; i < h->timed.size(); ++i) {
        if (h->timed[i].variant != variant) continue;
        SYMB_HIP(h, hipEventSynchronize(h->tev[2 * i + 1]));
        float ms = 0.f;
        SYMB_HIP(h, hipEventElapsedTime(&ms, h->tev[2 * i], h->tev[2 * i + 1]));
        *ms_total += ms;
        *launches += 1;
        *flops_total += h->timed[i].flops;
    }
    return SYMB_OK;
}

symb_status symb_destroy(symb_handle h) {
    if (!h) return SYMB_OK;
    (void)hipSetDevice(h->device);
    for (auto& e : h->tev) (void)hipEventDestroy(e);
    for (int i = 0; i < kSlots; ++i) {
        if (h->slot_used[i]) (void)hipEventSynchronize(h->slot_done[i]);
        if (h->slot_done[i]) (void)hipEventDestroy(h->slot_done[i]);
    }
    if (h->dev_ring) (void)hipFree(h->dev_ring);
    if (h->host_ring) (void)hipHostFree(h->host_ring);
    delete h;
    return SYMB_OK;
}

symb_status symb_validate_batch(const symb_batch* b) { return validate(nullptr, b); }

symb_status symb_debug_row_segment_map(const symb_batch* b, int32_t* host_out) {
    symb_status st = validate(nullptr, b);
    if (st != SYMB_OK) return st;
    if (!host_out && b->seg_offsets[b->num_segments] > 0) return fail(nullptr, SYMB_ERR_INVALID_ARG, "host_out is null");
    for (int i = 0; i < b->num_segments; ++i)
        for (int t = b->seg_offsets[i]; t < b->seg_offsets[i + 1]; ++t) host_out[t] = i;
    return SYMB_OK;
}

symb_status symb_plan_row_tiles(const symb_batch* b, int32_t tile_m, int32_t* seg_lo, int32_t* seg_hi, int32_t* num_tiles) {
    symb_status st = validate(nullptr, b);
    if (st != SYMB_OK) return st;
    if (tile_m <= 0 || !num_tiles) return fail(nullptr, SYMB_ERR_INVALID_ARG, "tile_m must be positive and num_tiles non-null");
    std::vector<int32_t> lo, hi;
    plan_row_tiles(b, tile_m, lo, hi);
    *num_tiles = (int32_t)lo.size();
    if (!lo.empty() && (!seg_lo || !seg_hi)) return fail(nullptr, SYMB_ERR_INVALID_ARG, "seg_lo / seg_hi is null");
    for (size_t u = 0; u < lo.size(); ++u) {
        seg_lo[u] = lo[u];
        seg_hi[u] = hi[u];
    }
    return SYMB_OK;
}

static bool wants_lora_grad(const symb_batch* b) {
    for (int i = 0; i < b->num_segments; ++i)
        if (b->adapters[i].kind == SYMB_ADAPTER_LORA && (b->adapters[i].dA || b->adapters[i].dB) &&
            b->seg_offsets[i + 1] > b->seg_offsets[i])
            return true;
    return false;
}

symb_status symb_workspace_bytes(const symb_batch* b, int32_t op, size_t* out) {
    symb_status st = validate(nullptr, b);
    if (st != SYMB_OK) return st;
    if (!out) return fail(nullptr, SYMB_ERR_INVALID_ARG, "out is null");
    if (op < SYMB_OP_FWD || op > SYMB_OP_BWD_INPUT_INPLACE) return fail(nullptr, SYMB_ERR_INVALID_ARG, "unknown op %d", op);
    const BatchInfo bi = inspect(b);
    const bool staged = op == SYMB_OP_FWD_INPLACE || op == SYMB_OP_BWD_INPUT_INPLACE;
    const int base_op = op == SYMB_OP_FWD_INPLACE ? SYMB_OP_FWD : op == SYMB_OP_BWD_INPUT_INPLACE ? SYMB_OP_BWD_INPUT : op;
    *out = ws_layout(b, bi, base_op, true, wants_lora_grad(b), staged).total;
    return SYMB_OK;
}

// ---------------------------------------------------------------------------------------------
// Checks a per-segment noise array (width = row length in elements) and turns it into device descriptors.
symb_status make_noisedesc(symb_handle h, const symb_batch* b, const symb_noise* noise, const char* what,
                           std::vector<NoiseDesc>& out) {
    out.assign(b->num_segments, NoiseDesc{nullptr, 0, 0});
    for (int i = 0; i < b->num_segments; ++i) {
        const symb_noise& n = noise[i];
        if (!n.ptr) continue;
        const int len = b->seg_offsets[i + 1] - b->seg_offsets[i];
        if (n.rows != 1 && n.rows != len)
            return fail(h, SYMB_ERR_INVALID_ARG, "%s of segment %d has %d rows: must be 1 or the segment's %d tokens", what, i, n.rows, len);
        if (misaligned16(n.ptr)) return fail(h, SYMB_ERR_INVALID_ARG, "%s of segment %d is not 16-byte aligned", what, i);
        out[i] = NoiseDesc{(const bf16*)n.ptr, n.rows, 0};
    }
    return SYMB_OK;
}

// Per-segment buffers (one DEVICE pointer per segment, HOST array): alignment, presence for
// non-empty segments, and, for the GEMM's activation operand, that they all lie inside one 4 GiB
// window (lane offsets are 32 bits wide).  *base receives the lowest address.
symb_status check_seg_ptrs(symb_handle h, const symb_batch* b, const void* const* seg, size_t row_bytes, const char* what,
                           bool need_window, const void** base) {
    uintptr_t lo = UINTPTR_MAX, hi = 0;
    for (int i = 0; i < b->num_segments; ++i) {
        const size_t n = (size_t)(b->seg_offsets[i + 1] - b->seg_offsets[i]);
        if (!n) continue;
        if (!seg[i]) return fail(h, SYMB_ERR_INVALID_ARG, "%s of segment %d is null", what, i);
        if (misaligned16(seg[i])) return fail(h, SYMB_ERR_INVALID_ARG, "%s of segment %d is not 16-byte aligned", what, i);
        lo = std::min(lo, (uintptr_t)seg[i]);
        hi = std::max(hi, (uintptr_t)seg[i] + n * row_bytes);
    }
    if (need_window && hi > lo && hi - lo > ((uint64_t)1 << 32) - 65536)
        return fail(h, SYMB_ERR_UNSUPPORTED, "%s buffers span %zu bytes: they must lie within one 4 GiB window", what, (size_t)(hi - lo));
    if (base) *base = (const void*)(lo == UINTPTR_MAX ? 0 : lo);
    return SYMB_OK;
}

// Whether any output buffer of a per-segment call shares bytes with any of its input buffers.
static bool seg_buffers_overlap(const symb_batch* b, const void* const* in_seg, size_t in_row_bytes, void* const* out_seg,
                                size_t out_row_bytes) {
    std::vector<std::pair<uintptr_t, uintptr_t>> in;
    for (int i = 0; i < b->num_segments; ++i) {
        const size_t n = (size_t)(b->seg_offsets[i + 1] - b->seg_offsets[i]);
        if (n) in.emplace_back((uintptr_t)in_seg[i], (uintptr_t)in_seg[i] + n * in_row_bytes);
    }
    std::sort(in.begin(), in.end());
    for (size_t k = 1; k < in.size(); ++k) in[k].second = std::max(in[k].second, in[k - 1].second);   // running end: sorted by start
    for (int i = 0; i < b->num_segments; ++i) {
        const size_t n = (size_t)(b->seg_offsets[i + 1] - b->seg_offsets[i]);
        if (!n) continue;
        const uintptr_t lo = (uintptr_t)out_seg[i], hi = lo + n * out_row_bytes;
        // the last input interval that starts before hi: with the running end it tells whether any reaches past lo
        auto it = std::lower_bound(in.begin(), in.end(), std::make_pair(hi, (uintptr_t)0));
        if (it != in.begin() && std::prev(it)->second > lo) return true;
    }
    return false;
}

static symb_status forward_impl(symb_handle h, const symb_batch* b, const void* X, const void* W, const void* bias,
                                const symb_noise* noise_effect, void* Y, void* Ybase, void* ws, size_t ws_bytes, void* stream,
                                const void* const* X_seg = nullptr, void* const* Y_seg = nullptr) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    CallGuard guard(h);
    if ((st = validate(h, b)) != SYMB_OK) return st;
    const BatchInfo bi = inspect(b);
    if (bi.T == 0) return SYMB_OK;
    const bool seg_io = X_seg != nullptr;
    const void* x_base = nullptr;
    if (seg_io) {
        if (!Y_seg || !W) return fail(h, SYMB_ERR_INVALID_ARG, "X_seg, Y_seg and W are required");
        // with an IA3_IN segment the GEMM reads a flat, scaled copy of the rows: no window needed then
        if ((st = check_seg_ptrs(h, b, X_seg, (size_t)b->d_in * 2, "X", bi.n_ia3in == 0, &x_base)) != SYMB_OK) return st;
        if ((st = check_seg_ptrs(h, b, (const void* const*)Y_seg, (size_t)b->d_out * 2, "Y", false, nullptr)) != SYMB_OK) return st;
    } else if (!X || !W || !Y) return fail(h, SYMB_ERR_INVALID_ARG, "X, W and Y are required");
    std::vector<NoiseDesc> nd;
    if (noise_effect && (st = make_noisedesc(h, b, noise_effect, "noise effect", nd)) != SYMB_OK) return st;
    if (misaligned16(X) || misaligned16(W) || misaligned16(Y) || misaligned16(Ybase) || misaligned16(bias) || misaligned16(ws))
        return fail(h, SYMB_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    // Per-segment buffers whose outputs overlap inputs (a client's one buffer used for both, Sec. 3.5):
    // column tiles of a row tile run at different times, so the GEMM writes a flat copy in the
    // workspace and a row scatter, after it on the stream, fills the clients' buffers.
    const bool staged = seg_io && seg_buffers_overlap(b, X_seg, (size_t)b->d_in * 2, Y_seg, (size_t)b->d_out * 2);
    const WsLayout wl = ws_layout(b, bi, SYMB_OP_FWD, true, false, staged);
    const size_t ws_need = wl.mandatory;     // the regions after it are optional
    if (ws_need > ws_bytes || (ws_need && !ws))
        return fail(h, SYMB_ERR_WORKSPACE_TOO_SMALL, "forward needs %zu workspace bytes, got %zu%s", ws_need, ws_bytes,
                    staged ? " (output buffers overlap input buffers: size the workspace with SYMB_OP_FWD_INPLACE)" : "");
    const SplitPlan ksp = gemm_split_plan(bi.T, b->d_out, b->d_in);
    const bool k_split = wl.tp_bytes && ws && ws_bytes >= wl.total && !Ybase && h->opt_k_split && h->xcd_rule;
    hipStream_t s = (hipStream_t)stream;

    const int bm = gemm_tile_m(bi.T, b->d_out);
    std::vector<int32_t> lo, hi;
    plan_row_tiles(b, bm, lo, hi);
    std::vector<RowChunk> chunks, all_chunks;
    plan_chunks(b, kSkinnyRows, SYMB_ADAPTER_LORA, chunks);
    // Input-major weight: the forward is the N-contiguous GEMM, whose LoRA steps read the adapter
    // side as [rank][d_out] rows: B_i^T, packed into the workspace; a second descriptor set points there.
    const bool conv1d = b->weight_layout == SYMB_WEIGHT_CONV1D;
    const bool small = small_path(h, bi.T, !conv1d, (long long)b->d_in * b->d_out, Ybase != nullptr, wl, ws, ws_bytes);
    const bool copy_rows = bi.n_ia3in > 0 || (small && seg_io);      // the product reads a flat copy of X (scaled / gathered)
    if (copy_rows || staged) plan_chunks(b, kSkinnyRows, -1, all_chunks);
    const std::vector<SegDesc> sd = make_segdesc(b);
    unsigned char* wsb = (unsigned char*)ws;
    std::vector<SegDesc> sd_gemm = sd;
    std::vector<int64_t> pk_off(bi.S, 0);
    if (conv1d && bi.n_lora) {
        int64_t cur = 0;
        for (int i = 0; i < bi.S; ++i)
            if (sd[i].kind == KIND_LORA) {
                pk_off[i] = cur;
                sd_gemm[i].A = (const bf16*)(wsb + wl.pk_off) + cur;
                cur += (int64_t)sd[i].rpad * b->d_out;
            }
    }
    Blob blob;
    const size_t o_seg = blob.add(sd.data(), sd.size());
    const size_t o_segg = blob.add(sd_gemm.data(), sd_gemm.size());
    const size_t o_off = blob.add(b->seg_offsets, (size_t)bi.S + 1);
    const size_t o_lo = blob.add(lo.data(), lo.size());
    const size_t o_hi = blob.add(hi.data(), hi.size());
    const std::vector<int32_t> tile_epi = plan_tile_kind(b, lo, hi, SYMB_ADAPTER_IA3);
    const size_t o_te = blob.add(tile_epi.data(), tile_epi.size());
    const size_t o_ch = blob.add(chunks.data(), chunks.size());
    const size_t o_nd = blob.add(nd.data(), nd.size());
    const size_t o_pk = blob.add(pk_off.data(), pk_off.size());
    const size_t o_all = blob.add(all_chunks.data(), all_chunks.size());
    const size_t o_xs = blob.add(X_seg, seg_io ? (size_t)bi.S : 0);
    const size_t o_ys = blob.add(Y_seg, seg_io ? (size_t)bi.S : 0);
    const std::vector<int32_t> k_zero(k_split ? ksp.slots : 0, 0);
    const size_t o_kc = blob.add(k_zero.data(), k_zero.size());   // arrival counters of the K-split tiles
    unsigned char* dev = nullptr;
    if ((st = upload(h, blob, s, &dev)) != SYMB_OK) return st;

    // IA3 input scaling: the GEMM multiplies a copy of X whose IA3_IN rows are scaled by l_i
    // (LoRA segments, if any, still shrink the caller's X: their rows are not touched by the copy)
    const bf16* x_op = (const bf16*)X;
    if (copy_rows) {
        bf16* const copy = (bf16*)(wsb + (bi.n_ia3in ? wl.sc_off : wl.sg_off));
        ScaleParams sc{(const bf16*)X, copy, b->d_in, (const RowChunk*)(dev + o_all),
                       (const SegDesc*)(dev + o_seg), KIND_IA3_IN, seg_io ? (const bf16* const*)(dev + o_xs) : nullptr,
                       (const int32_t*)(dev + o_off)};
        if (!all_chunks.empty()) {
            hipLaunchKernelGGL(symb_ia3_scale_rows_kernel, dim3((unsigned)all_chunks.size()), dim3(256), 0, s, sc);
            SYMB_HIP(h, hipGetLastError());
        }
        x_op = copy;
    }
    bf16* Hs = bi.n_lora ? (bf16*)(wsb + wl.h_off) : nullptr;
    if (conv1d && bi.n_lora && !small) {
        PackParams pp{(const SegDesc*)(dev + o_seg), (bf16*)(wsb + wl.pk_off), (const int64_t*)(dev + o_pk), b->d_out};
        hipLaunchKernelGGL(symb_pack_bt_kernel, dim3((b->d_out + 255) / 256, bi.S), dim3(256), 0, s, pp);
        SYMB_HIP(h, hipGetLastError());
    }
    if (bi.n_lora) {
        SkinnyParams sp{};
        sp.L = (const bf16*)X;
        sp.out = Hs;
        sp.K = b->d_in;
        sp.out_pitch = 2 * bi.max_rpad;
        sp.chunks = (const RowChunk*)(dev + o_ch);
        sp.seg = (const SegDesc*)(dev + o_seg);
        sp.use_packed = 0;
        if (seg_io) {
            sp.L_seg = (const bf16* const*)(dev + o_xs);
            sp.off = (const int32_t*)(dev + o_off);
        }
        if ((st = launch_skinny(h, sp, (int)chunks.size(), bi.max_rpad, s)) != SYMB_OK) return st;
    }
    // A handful of rows (decode steps): the weight-streaming kernels instead of the tiled GEMM.  Measured
    // against the tiled kernel with its K-split (33-40 us per call from 4 to 64 rows): 17-20 us up to 16 rows on
    // 4096 x 4096 (descriptors in place), but slower from 24 rows on.
    if (small) {
        SmallEpilogue ep{};
        ep.C = (bf16*)Y;
        ep.Cbase = (bf16*)Ybase;
        ep.c_seg = seg_io ? (bf16* const*)(dev + o_ys) : nullptr;
        ep.bias = (const bf16*)bias;
        ep.N = b->d_out;
        ep.T = bi.T;
        ep.S = bi.S;
        ep.off = (const int32_t*)(dev + o_off);
        ep.seg = (const SegDesc*)(dev + o_seg);
        ep.ext = Hs;
        ep.ext_pitch = 2 * bi.max_rpad;
        ep.backward = 0;
        ep.lora_term = 1;
        ep.neff = nd.empty() ? nullptr : (const NoiseDesc*)(dev + o_nd);
        if ((st = launch_small(h, x_op, (const bf16*)W, !conv1d, b->d_in, ep, (float*)(wsb + wl.sp_off), s)) != SYMB_OK) return st;
        { guard.completed = true; return seal_slot(h, s); }
    }
    GemmParams gp{};
    gp.Aop = x_op;
    if (seg_io) {
        if (!copy_rows) {          // (a flat copy of the rows, scaled for IA3_IN, is read as one tensor)
            gp.Aop = nullptr;
            gp.a_seg = (const bf16* const*)(dev + o_xs);
            gp.a_base = (const bf16*)x_base;
        }
        if (!staged) gp.c_seg = (bf16* const*)(dev + o_ys);
    }
    gp.Bop = (const bf16*)W;
    gp.C = staged ? (bf16*)(wsb + wl.so_off) : (bf16*)Y;
    gp.Cbase = (bf16*)Ybase;
    gp.bias = (const bf16*)bias;
    gp.M = bi.T;
    gp.N = b->d_out;
    gp.K = b->d_in;
    gp.off = (const int32_t*)(dev + o_off);
    gp.seg = (const SegDesc*)(dev + o_segg);
    gp.tile_seg_lo = (const int32_t*)(dev + o_lo);
    gp.tile_seg_hi = (const int32_t*)(dev + o_hi);
    gp.ext = Hs;
    gp.ext_pitch = 2 * bi.max_rpad;
    gp.epi_ia3 = bi.n_ia3 > 0 ? KIND_IA3 : 0;
    gp.tile_epi = (const int32_t*)(dev + o_te);
    gp.neff = nd.empty() ? nullptr : (const NoiseDesc*)(dev + o_nd);
    gp.timing_flops = gemm_flops(b, b->d_out, b->d_in, bi.n_lora > 0);
    gp.group_m = gemm_group_m((bi.T + bm - 1) / bm, (b->d_out + bm - 1) / bm, lo, hi);
    if (k_split) {
        gp.k_parts = ksp.parts;
        gp.k_whole = ksp.whole;
        gp.partial = (float*)(wsb + wl.tp_off);
        gp.k_count = (int*)(dev + o_kc);
    }
    // W [d_out][d_in]: K-contiguous weight rows.  W [d_in][d_out]: the weight is the [K][N] operand.
    st = conv1d ? launch_gemm<true>(h, gp, s) : launch_gemm<false>(h, gp, s);
    if (st != SYMB_OK) return st;
    if (staged) {
        ScatterParams sc{(const bf16*)(wsb + wl.so_off), b->d_out, (const RowChunk*)(dev + o_all), (bf16* const*)(dev + o_ys),
                         (const int32_t*)(dev + o_off)};
        hipLaunchKernelGGL(symb_scatter_rows_kernel, dim3((unsigned)all_chunks.size()), dim3(256), 0, s, sc);
        SYMB_HIP(h, hipGetLastError());
    }
    { guard.completed = true; return seal_slot(h, s); }
}

symb_status symb_base_linear_fwd(symb_handle h, const symb_batch* b, const void* X, const void* W, const void* bias,
                                 void* Y, void* Ybase, void* ws, size_t ws_bytes, void* stream) {
    return forward_impl(h, b, X, W, bias, nullptr, Y, Ybase, ws, ws_bytes, stream);
}

// The forward with its workspace in the file-scope scratch array of this device: no device allocation
// by the library or the caller.  Same kernels and launches as symb_base_linear_fwd.
symb_status symb_base_linear_fwd_static(symb_handle h, const symb_batch* b, const void* X, const void* W, const void* bias,
                                        void* Y, void* Ybase, void* stream) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if ((st = validate(h, b)) != SYMB_OK) return st;
    const BatchInfo bi = inspect(b);
    const WsLayout wl = ws_layout(b, bi, SYMB_OP_FWD, true, false);
    const size_t need = wl.mandatory;        // the optional regions (small-batch kernels, K-split partial tiles) are used only if they fit too
    if (need > (size_t)SYMB_STATIC_SCRATCH_BYTES)
        return fail(h, SYMB_ERR_WORKSPACE_TOO_SMALL, "this batch needs %zu bytes of workspace; the static scratch array holds %zu "
                    "(use symb_base_linear_fwd with a workspace of the caller's)", need, (size_t)SYMB_STATIC_SCRATCH_BYTES);
    return forward_impl(h, b, X, W, bias, nullptr, Y, Ybase, h->static_scratch, (size_t)SYMB_STATIC_SCRATCH_BYTES, stream);
}

symb_status symb_base_linear_fwd_seg(symb_handle h, const symb_batch* b, const void* const* X_seg, const void* W,
                                     const void* bias, void* const* Y_seg, void* ws, size_t ws_bytes, void* stream) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (!X_seg || !Y_seg) return fail(h, SYMB_ERR_INVALID_ARG, "X_seg and Y_seg are required");
    return forward_impl(h, b, nullptr, W, bias, nullptr, nullptr, nullptr, ws, ws_bytes, stream, X_seg, Y_seg);
}

symb_status symb_base_linear_fwd_denoise(symb_handle h, const symb_batch* b, const void* Xn, const void* W, const void* bias,
                                         const symb_noise* noise_effect, void* Y, void* ws, size_t ws_bytes, void* stream) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (!noise_effect) return fail(h, SYMB_ERR_INVALID_ARG, "noise_effect is required");
    return forward_impl(h, b, Xn, W, bias, noise_effect, Y, nullptr, ws, ws_bytes, stream);
}

symb_status symb_noise_add(symb_handle h, const symb_batch* b, const void* X, const symb_noise* noise, void* Xn, void* stream) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    CallGuard guard(h);
    if ((st = validate(h, b)) != SYMB_OK) return st;
    if (!noise) return fail(h, SYMB_ERR_INVALID_ARG, "noise is required");
    const BatchInfo bi = inspect(b);
    if (bi.T == 0) return SYMB_OK;
    if (!X || !Xn) return fail(h, SYMB_ERR_INVALID_ARG, "X and Xn are required");
    if (misaligned16(X) || misaligned16(Xn)) return fail(h, SYMB_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    std::vector<NoiseDesc> nd;
    if ((st = make_noisedesc(h, b, noise, "noise", nd)) != SYMB_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    std::vector<RowChunk> chunks;
    plan_chunks(b, kSkinnyRows, -1, chunks);
    Blob blob;
    const size_t o_off = blob.add(b->seg_offsets, (size_t)bi.S + 1);
    const size_t o_ch = blob.add(chunks.data(), chunks.size());
    const size_t o_nd = blob.add(nd.data(), nd.size());
    unsigned char* dev = nullptr;
    if ((st = upload(h, blob, s, &dev)) != SYMB_OK) return st;
    NoiseAddParams np{(const bf16*)X, (bf16*)Xn, b->d_in, (const RowChunk*)(dev + o_ch), (const int32_t*)(dev + o_off),
                      (const NoiseDesc*)(dev + o_nd)};
    hipLaunchKernelGGL(symb_noise_add_kernel, dim3((unsigned)chunks.size()), dim3(256), 0, s, np);
    SYMB_HIP(h, hipGetLastError());
    { guard.completed = true; return seal_slot(h, s); }
}

// ---------------------------------------------------------------------------------------------
static symb_status backward_input_impl(symb_handle h, const symb_batch* b, const void* dY, const void* W, void* dX,
                                       void* dXbase, uint32_t flags, void* ws, size_t ws_bytes, void* stream,
                                       const void* const* dY_seg, void* const* dX_seg);

symb_status symb_base_linear_bwd_input(symb_handle h, const symb_batch* b, const void* dY, const void* W, void* dX,
                                       uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
    return backward_input_impl(h, b, dY, W, dX, nullptr, flags, ws, ws_bytes, stream, nullptr, nullptr);
}

symb_status symb_base_linear_bwd_input_ex(symb_handle h, const symb_batch* b, const void* dY, const void* W, void* dX,
                                          void* dXbase, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
    return backward_input_impl(h, b, dY, W, dX, dXbase, flags, ws, ws_bytes, stream, nullptr, nullptr);
}

symb_status symb_base_linear_bwd_input_seg(symb_handle h, const symb_batch* b, const void* const* dY_seg, const void* W,
                                           void* const* dX_seg, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (!dY_seg || !dX_seg) return fail(h, SYMB_ERR_INVALID_ARG, "dY_seg and dX_seg are required");
    return backward_input_impl(h, b, nullptr, W, nullptr, nullptr, flags, ws, ws_bytes, stream, dY_seg, dX_seg);
}

static symb_status backward_input_impl(symb_handle h, const symb_batch* b, const void* dY, const void* W, void* dX,
                                       void* dXbase, uint32_t flags, void* ws, size_t ws_bytes, void* stream,
                                       const void* const* dY_seg, void* const* dX_seg) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    CallGuard guard(h);
    if ((st = validate(h, b)) != SYMB_OK) return st;
    if (flags & ~(uint32_t)(SYMB_BWD_BASE_ONLY | SYMB_BWD_REUSE_DH)) return fail(h, SYMB_ERR_INVALID_ARG, "unknown backward flag %u", flags);
    if ((flags & SYMB_BWD_BASE_ONLY) && (flags & SYMB_BWD_REUSE_DH))
        return fail(h, SYMB_ERR_INVALID_ARG, "SYMB_BWD_REUSE_DH makes no sense with SYMB_BWD_BASE_ONLY");
    const bool take_dh = (flags & SYMB_BWD_REUSE_DH) != 0;      // dH is in the workspace already (a gradient call on this batch left it)
    const BatchInfo bi = inspect(b);
    if (bi.T == 0) return SYMB_OK;
    const bool seg_io = dY_seg != nullptr;
    const void* g_base = nullptr;
    if (seg_io) {
        if (!W) return fail(h, SYMB_ERR_INVALID_ARG, "W is required");
        const bool copy_first = !(flags & SYMB_BWD_BASE_ONLY) && bi.n_ia3 > 0;     // then the GEMM reads the scaled copy, not the buffers
        if ((st = check_seg_ptrs(h, b, dY_seg, (size_t)b->d_out * 2, "dY", !copy_first, &g_base)) != SYMB_OK) return st;
        if ((st = check_seg_ptrs(h, b, (const void* const*)dX_seg, (size_t)b->d_in * 2, "dX", false, nullptr)) != SYMB_OK) return st;
    } else if (!dY || !W || !dX) return fail(h, SYMB_ERR_INVALID_ARG, "dY, W and dX are required");
    if (misaligned16(dY) || misaligned16(W) || misaligned16(dX) || misaligned16(dXbase) || misaligned16(ws))
        return fail(h, SYMB_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const bool full = !(flags & SYMB_BWD_BASE_ONLY);
    const bool staged = seg_io && seg_buffers_overlap(b, dY_seg, (size_t)b->d_out * 2, dX_seg, (size_t)b->d_in * 2);   // see the forward
    const WsLayout wl = ws_layout(b, bi, SYMB_OP_BWD_INPUT, full, false, staged);
    const size_t ws_need = wl.mandatory;     // the regions after it are optional
    if (ws_need > ws_bytes || (ws_need && !ws))
        return fail(h, SYMB_ERR_WORKSPACE_TOO_SMALL, "backward needs %zu workspace bytes, got %zu%s", ws_need, ws_bytes,
                    staged ? " (output buffers overlap input buffers: size the workspace with SYMB_OP_BWD_INPUT_INPLACE)" : "");
    const SplitPlan ksp = gemm_split_plan(bi.T, b->d_in, b->d_out);
    const bool k_split = wl.tp_bytes && ws && ws_bytes >= wl.total && !dXbase && h->opt_k_split && h->xcd_rule;
    hipStream_t s = (hipStream_t)stream;
    const bool lora = full && bi.n_lora > 0, ia3 = full && bi.n_ia3 > 0;
    const bool conv1d_early = b->weight_layout == SYMB_WEIGHT_CONV1D;

    const int bm = gemm_tile_m(bi.T, b->d_in);
    std::vector<int32_t> lo, hi;
    plan_row_tiles(b, bm, lo, hi);
    std::vector<RowChunk> chunks, all_chunks;
    if (lora) plan_chunks(b, kSkinnyRows, SYMB_ADAPTER_LORA, chunks);
    // Rows of IA3 segments enter the GEMM scaled by l_i: a scaled copy of those rows goes to the
    // workspace, and the GEMM takes every row from where it lies (per-row base pointers: the copy for
    // IA3 rows, the caller's dY for the others).  Lane offsets are 32 bits wide, so this needs all those
    // rows within one 4 GiB window; failing that, all rows are copied and the GEMM reads the copy alone.
    unsigned char* const wsb0 = (unsigned char*)ws;
    std::vector<const void*> mix;           // per segment: where the GEMM reads its rows
    bool ia3_mixed = false;
    // a handful of rows: the weight-streaming kernels, which read one flat copy of the rows (gathered from
    // per-segment buffers, IA3 rows scaled) in the workspace
    const bool small = small_path(h, bi.T, conv1d_early, (long long)b->d_in * b->d_out, dXbase != nullptr, wl, ws, ws_bytes);
    const bool small_copy = small && (seg_io || ia3);
    if (small_copy) {
        plan_chunks(b, kSkinnyRows, -1, all_chunks);
    } else if (ia3) {
        mix.assign(bi.S, nullptr);
        uintptr_t lo_a = UINTPTR_MAX, hi_a = 0;
        for (int i = 0; i < bi.S; ++i) {
            const size_t n = (size_t)(b->seg_offsets[i + 1] - b->seg_offsets[i]), row_bytes = (size_t)b->d_out * 2;
            if (!n) continue;
            const unsigned char* src = b->adapters[i].kind == SYMB_ADAPTER_IA3
                                           ? wsb0 + wl.sc_off + (size_t)b->seg_offsets[i] * row_bytes
                                           : (seg_io ? (const unsigned char*)dY_seg[i] : (const unsigned char*)dY + (size_t)b->seg_offsets[i] * row_bytes);
            mix[i] = src;
            lo_a = std::min(lo_a, (uintptr_t)src);
            hi_a = std::max(hi_a, (uintptr_t)src + n * row_bytes);
        }
        ia3_mixed = hi_a > lo_a && hi_a - lo_a <= ((uint64_t)1 << 32) - 65536;
        if (ia3_mixed) g_base = (const void*)lo_a;
        plan_chunks(b, kSkinnyRows, ia3_mixed ? (int)SYMB_ADAPTER_IA3 : -1, all_chunks);
    }
    const std::vector<SegDesc> sd = make_segdesc(b);
    unsigned char* wsb = (unsigned char*)ws;
    // Input-major weight: the input gradient is the K-contiguous GEMM (W rows are d_out long),
    // whose LoRA steps read the adapter side as [d_in][rank] rows: A_i^T, packed into the workspace.
    const bool conv1d = b->weight_layout == SYMB_WEIGHT_CONV1D;
    std::vector<SegDesc> sd_gemm = sd;
    std::vector<int64_t> pk_off(bi.S, 0), pa_off(bi.S, 0);
    {
        int64_t cur = 0, cura = 0;
        for (int i = 0; i < bi.S; ++i)
            if (sd[i].kind == KIND_LORA) {
                pk_off[i] = cur;
                cur += (int64_t)sd[i].rpad * b->d_out;
                if (conv1d && lora) {
                    pa_off[i] = cura;
                    sd_gemm[i].B = (const bf16*)(wsb + wl.pa_off) + cura;
                    cura += (int64_t)align_up((size_t)sd[i].rank * b->d_in, 8);
                }
            }
    }
    Blob blob;
    const size_t o_seg = blob.add(sd.data(), sd.size());
    const size_t o_segg = blob.add(sd_gemm.data(), sd_gemm.size());
    const size_t o_off = blob.add(b->seg_offsets, (size_t)bi.S + 1);
    const size_t o_lo = blob.add(lo.data(), lo.size());
    const size_t o_hi = blob.add(hi.data(), hi.size());
    const std::vector<int32_t> tile_epi = plan_tile_kind(b, lo, hi, SYMB_ADAPTER_IA3_IN);
    const size_t o_te = blob.add(tile_epi.data(), tile_epi.size());
    const size_t o_ch = blob.add(chunks.data(), chunks.size());
    const size_t o_all = blob.add(all_chunks.data(), all_chunks.size());
    const size_t o_pk = blob.add(pk_off.data(), pk_off.size());
    const size_t o_pa = blob.add(pa_off.data(), pa_off.size());
    const size_t o_gs = blob.add(dY_seg, seg_io ? (size_t)bi.S : 0);
    const size_t o_xs = blob.add(dX_seg, seg_io ? (size_t)bi.S : 0);
    const size_t o_mix = blob.add(mix.data(), ia3_mixed ? mix.size() : 0);
    std::vector<RowChunk> row_chunks;
    if (staged) plan_chunks(b, kSkinnyRows, -1, row_chunks);
    const size_t o_rows = blob.add(row_chunks.data(), row_chunks.size());
    const std::vector<int32_t> k_zero(k_split ? ksp.slots : 0, 0);
    const size_t o_kc = blob.add(k_zero.data(), k_zero.size());   // arrival counters of the K-split tiles
    unsigned char* dev = nullptr;
    if ((st = upload(h, blob, s, &dev)) != SYMB_OK) return st;

    const bf16* a_op = (const bf16*)dY;
    bf16* dH = nullptr;
    if (lora && conv1d && !small) {
        PackAtParams pa{(const SegDesc*)(dev + o_seg), (bf16*)(wsb + wl.pa_off), (const int64_t*)(dev + o_pa), b->d_in};
        hipLaunchKernelGGL(symb_pack_at_kernel, dim3((b->d_in + 255) / 256, bi.S), dim3(256), 0, s, pa);
        SYMB_HIP(h, hipGetLastError());
    }
    if (lora) dH = (bf16*)(wsb + wl.dh_off);
    if (lora && !take_dh) {
        PackParams pp{(const SegDesc*)(dev + o_seg), (bf16*)(wsb + wl.pk_off), (const int64_t*)(dev + o_pk), b->d_out};
        hipLaunchKernelGGL(symb_pack_bt_kernel, dim3((b->d_out + 255) / 256, bi.S), dim3(256), 0, s, pp);
        SYMB_HIP(h, hipGetLastError());
        SkinnyParams sp{};
        sp.L = (const bf16*)dY;
        sp.out = dH;
        sp.K = b->d_out;
        sp.out_pitch = 2 * bi.max_rpad;
        sp.chunks = (const RowChunk*)(dev + o_ch);
        sp.seg = (const SegDesc*)(dev + o_seg);
        sp.packed = (const bf16*)(wsb + wl.pk_off);
        sp.packed_off = (const int64_t*)(dev + o_pk);
        sp.use_packed = 1;
        if (seg_io) {
            sp.L_seg = (const bf16* const*)(dev + o_gs);
            sp.off = (const int32_t*)(dev + o_off);
        }
        if ((st = launch_skinny(h, sp, (int)chunks.size(), bi.max_rpad, s)) != SYMB_OK) return st;
    }
    bool a_from_seg = seg_io;
    if (ia3 || small_copy) {
        a_from_seg = ia3_mixed;
        bf16* const copy = (bf16*)(wsb + (small_copy ? wl.sg_off : wl.sc_off));
        ScaleParams sc{(const bf16*)dY, copy, b->d_out, (const RowChunk*)(dev + o_all), (const SegDesc*)(dev + o_seg),
                       ia3 ? (int)KIND_IA3 : -1, seg_io ? (const bf16* const*)(dev + o_gs) : nullptr, (const int32_t*)(dev + o_off)};
        if (!all_chunks.empty()) {          // (every IA3 segment of the batch may be empty: nothing to scale then)
            hipLaunchKernelGGL(symb_ia3_scale_rows_kernel, dim3((unsigned)all_chunks.size()), dim3(256), 0, s, sc);
            SYMB_HIP(h, hipGetLastError());
        }
        a_op = copy;
    }
    if (small) {
        SmallEpilogue ep{};
        ep.C = (bf16*)dX;
        ep.Cbase = (bf16*)dXbase;
        ep.c_seg = seg_io ? (bf16* const*)(dev + o_xs) : nullptr;
        ep.N = b->d_in;
        ep.T = bi.T;
        ep.S = bi.S;
        ep.off = (const int32_t*)(dev + o_off);
        ep.seg = (const SegDesc*)(dev + o_seg);
        ep.ext = dH;
        ep.ext_pitch = 2 * bi.max_rpad;
        ep.backward = 1;
        ep.lora_term = full ? 1 : 0;
        // W [d_out][d_in] is the [K][N] operand of dX = dY W; an input-major weight [d_in][d_out] is [N][K]
        if ((st = launch_small(h, a_op, (const bf16*)W, conv1d, b->d_out, ep, (float*)(wsb + wl.sp_off), s)) != SYMB_OK) return st;
        { guard.completed = true; return seal_slot(h, s); }
    }
    GemmParams gp{};
    gp.Aop = a_op;
    gp.Bop = (const bf16*)W;
    gp.C = (bf16*)dX;
    gp.Cbase = (bf16*)dXbase;
    if (a_from_seg) {
        gp.Aop = nullptr;
        gp.a_seg = (const bf16* const*)(dev + (ia3_mixed ? o_mix : o_gs));
        gp.a_base = (const bf16*)g_base;
    }
    if (seg_io && !staged) gp.c_seg = (bf16* const*)(dev + o_xs);
    if (staged) gp.C = (bf16*)(wsb + wl.so_off);
    gp.M = bi.T;
    gp.N = b->d_in;
    gp.K = b->d_out;
    gp.off = (const int32_t*)(dev + o_off);
    gp.seg = (const SegDesc*)(dev + o_segg);
    gp.tile_seg_lo = (const int32_t*)(dev + o_lo);
    gp.tile_seg_hi = (const int32_t*)(dev + o_hi);
    gp.ext = dH;
    gp.ext_pitch = 2 * bi.max_rpad;
    gp.epi_ia3 = (full && bi.n_ia3in > 0) ? KIND_IA3_IN : 0;      // dX rows of IA3_IN segments: l_i * (dY W)
    gp.tile_epi = (const int32_t*)(dev + o_te);
    gp.timing_flops = gemm_flops(b, b->d_in, b->d_out, lora);
    gp.group_m = gemm_group_m((bi.T + bm - 1) / bm, (b->d_in + bm - 1) / bm, lo, hi);
    if (k_split) {
        gp.k_parts = ksp.parts;
        gp.k_whole = ksp.whole;
        gp.partial = (float*)(wsb + wl.tp_off);
        gp.k_count = (int*)(dev + o_kc);
    }
    // W [d_out][d_in] is the [K][N] operand of dX = dY W; W [d_in][d_out] gives K-contiguous rows.
    st = conv1d ? launch_gemm<false>(h, gp, s) : launch_gemm<true>(h, gp, s);
    if (st != SYMB_OK) return st;
    if (staged) {
        ScatterParams sc{(const bf16*)(wsb + wl.so_off), b->d_in, (const RowChunk*)(dev + o_rows), (bf16* const*)(dev + o_xs),
                         (const int32_t*)(dev + o_off)};
        hipLaunchKernelGGL(symb_scatter_rows_kernel, dim3((unsigned)row_chunks.size()), dim3(256), 0, s, sc);
        SYMB_HIP(h, hipGetLastError());
    }
    { guard.completed = true; return seal_slot(h, s); }
}

// ---------------------------------------------------------------------------------------------
static symb_status adapter_grad_impl(symb_handle h, const symb_batch* b, const void* X, const void* dY, const void* Ybase,
                                     const void* dXbase, uint32_t flags, void* ws, size_t ws_bytes, void* stream,
                                     const void* const* X_seg, const void* const* dY_seg, const void* const* Ybase_seg);

symb_status symb_adapter_grad(symb_handle h, const symb_batch* b, const void* X, const void* dY, const void* Ybase,
                              uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
    return adapter_grad_impl(h, b, X, dY, Ybase, nullptr, flags, ws, ws_bytes, stream, nullptr, nullptr, nullptr);
}

symb_status symb_adapter_grad_ex(symb_handle h, const symb_batch* b, const void* X, const void* dY, const void* Ybase,
                                 const void* dXbase, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
    return adapter_grad_impl(h, b, X, dY, Ybase, dXbase, flags, ws, ws_bytes, stream, nullptr, nullptr, nullptr);
}

symb_status symb_adapter_grad_seg(symb_handle h, const symb_batch* b, const void* const* X_seg, const void* const* dY_seg,
                                  const void* const* Ybase_seg, uint32_t flags, void* ws, size_t ws_bytes, void* stream) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    if (!X_seg || !dY_seg) return fail(h, SYMB_ERR_INVALID_ARG, "X_seg and dY_seg are required");
    return adapter_grad_impl(h, b, nullptr, nullptr, nullptr, nullptr, flags, ws, ws_bytes, stream, X_seg, dY_seg, Ybase_seg);
}

static symb_status adapter_grad_impl(symb_handle h, const symb_batch* b, const void* X, const void* dY, const void* Ybase,
                                     const void* dXbase, uint32_t flags, void* ws, size_t ws_bytes, void* stream,
                                     const void* const* X_seg, const void* const* dY_seg, const void* const* Ybase_seg) {
    symb_status st = check_handle(h);
    if (st != SYMB_OK) return st;
    CallGuard guard(h);
    if ((st = validate(h, b)) != SYMB_OK) return st;
    if (flags & ~(uint32_t)(SYMB_GRAD_ACCUMULATE | SYMB_GRAD_REUSE_DH | SYMB_GRAD_REUSE_HS))
        return fail(h, SYMB_ERR_INVALID_ARG, "unknown gradient flag %u", flags);
    const bool reuse_dh = (flags & SYMB_GRAD_REUSE_DH) != 0, reuse_hs = (flags & SYMB_GRAD_REUSE_HS) != 0;
    const BatchInfo bi = inspect(b);
    const bool seg_io = X_seg != nullptr;
    if (seg_io) {
        if ((st = check_seg_ptrs(h, b, X_seg, (size_t)b->d_in * 2, "X", false, nullptr)) != SYMB_OK) return st;
        if ((st = check_seg_ptrs(h, b, dY_seg, (size_t)b->d_out * 2, "dY", false, nullptr)) != SYMB_OK) return st;
        if (Ybase_seg) {
            // what the client kept for dl: the pre-adapter output rows (IA3), the input gradient before the input scale (IA3_IN)
            for (int i = 0; i < bi.S; ++i) {
                const int k = b->adapters[i].kind;
                if ((k == SYMB_ADAPTER_IA3 || k == SYMB_ADAPTER_IA3_IN) && b->adapters[i].dA && b->seg_offsets[i + 1] > b->seg_offsets[i] &&
                    (!Ybase_seg[i] || misaligned16(Ybase_seg[i])))
                    return fail(h, SYMB_ERR_INVALID_ARG, "the saved rows of IA3 segment %d are null or misaligned", i);
            }
        }
    } else if (!X || !dY) {
        if (bi.T > 0) return fail(h, SYMB_ERR_INVALID_ARG, "X and dY are required");
    }
    if (misaligned16(X) || misaligned16(dY) || misaligned16(Ybase) || misaligned16(dXbase) || misaligned16(ws))
        return fail(h, SYMB_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const bool acc = (flags & SYMB_GRAD_ACCUMULATE) != 0;
    hipStream_t s = (hipStream_t)stream;

    // Which segments want which gradient.  Empty segments: zeros when overwriting, nothing otherwise.
    std::vector<int32_t> want_a, want_b, want_l, want_lin;
    std::vector<std::pair<float*, size_t>> zero_fill;
    int grad_max_rpad = 0;
    for (int i = 0; i < bi.S; ++i) {
        const symb_adapter& a = b->adapters[i];
        const bool empty = b->seg_offsets[i + 1] == b->seg_offsets[i];
        if (a.kind == SYMB_ADAPTER_LORA) {
            if (empty) {
                if (!acc && a.dA) zero_fill.emplace_back((float*)a.dA, (size_t)a.rank * b->d_in);
                if (!acc && a.dB) zero_fill.emplace_back((float*)a.dB, (size_t)a.rank * b->d_out);
                continue;
            }
            if (a.dA) want_a.push_back(i);
            if (a.dB) want_b.push_back(i);
            if (a.dA || a.dB) grad_max_rpad = std::max(grad_max_rpad, rpad_of(a.rank));
        } else if (a.kind == SYMB_ADAPTER_IA3 && a.dA) {
            if (empty) {
                if (!acc) zero_fill.emplace_back((float*)a.dA, (size_t)b->d_out);
                continue;
            }
            want_l.push_back(i);
        } else if (a.kind == SYMB_ADAPTER_IA3_IN && a.dA) {
            if (empty) {
                if (!acc) zero_fill.emplace_back((float*)a.dA, (size_t)b->d_in);
                continue;
            }
            want_lin.push_back(i);
        }
    }
    if (!want_lin.empty() && !(seg_io ? (const void*)Ybase_seg : dXbase))
        return fail(h, SYMB_ERR_INVALID_ARG, "an IA3_IN segment wants dl but dXbase (the input gradient before the input scale) is null");
    if (!want_l.empty() && !(seg_io ? (const void*)Ybase_seg : Ybase))
        return fail(h, SYMB_ERR_INVALID_ARG, "an IA3 segment wants dl but Ybase (the pre-adapter output) is null");
    const bool any_lora = !want_a.empty() || !want_b.empty();
    const WsLayout wl = ws_layout(b, bi, SYMB_OP_ADAPTER_GRAD, true, any_lora);
    if (wl.total > ws_bytes || (wl.total && !ws))
        return fail(h, SYMB_ERR_WORKSPACE_TOO_SMALL, "adapter_grad needs %zu workspace bytes, got %zu", wl.total, ws_bytes);
    // zeros of the empty segments: fill kernels, not memset nodes (safe under graph capture); enqueued
    // only once nothing before the launches can fail any more
    auto fill_zeros = [&]() -> symb_status {
        for (const auto& z : zero_fill) {
            hipLaunchKernelGGL(symb_fill_zero_kernel, dim3((unsigned)std::min<size_t>((z.second + 255) / 256, 1024)), dim3(256), 0, s, z.first, z.second);
            SYMB_HIP(h, hipGetLastError());
        }
        return SYMB_OK;
    };
    if (!any_lora && want_l.empty() && want_lin.empty()) return fill_zeros();

    // Row chunks of the LoRA segments that want a gradient (Hs for dB, dH for dA).
    std::vector<RowChunk> ch_h, ch_dh;
    for (int i : want_b)
        for (int r = b->seg_offsets[i]; r < b->seg_offsets[i + 1]; r += kSkinnyRows)
            ch_h.push_back(RowChunk{i, r, std::min(kSkinnyRows, b->seg_offsets[i + 1] - r), 0});
    for (int i : want_a)
        for (int r = b->seg_offsets[i]; r < b->seg_offsets[i + 1]; r += kSkinnyRows)
            ch_dh.push_back(RowChunk{i, r, std::min(kSkinnyRows, b->seg_offsets[i + 1] - r), 0});
    const std::vector<SegDesc> sd = make_segdesc(b);
    std::vector<int64_t> pk_off(bi.S, 0);
    {
        int64_t cur = 0;
        for (int i = 0; i < bi.S; ++i)
            if (sd[i].kind == KIND_LORA) {
                pk_off[i] = cur;
                cur += (int64_t)sd[i].rpad * b->d_out;
            }
    }
    // Work items of the two gradient launches: whole segments, or the runs of long ones (see grad_runs).
    auto plan_items = [&](const std::vector<int32_t>& want, int ncols, std::vector<GradItem>& items, std::vector<GradReduceItem>& red) {
        int64_t cur = 0;
        for (int i : want) {
            const int lo = b->seg_offsets[i], hi = b->seg_offsets[i + 1], runs = grad_runs(hi - lo);
            if (runs == 1) {
                items.push_back(GradItem{i, lo, hi, 1, 0});
                continue;
            }
            const int64_t n = (int64_t)b->adapters[i].rank * ncols;
            red.push_back(GradReduceItem{i, runs, cur});
            for (int q = 0; q < runs; ++q, cur += n)
                items.push_back(GradItem{i, lo + q * GRAD_SPLIT, std::min(hi, lo + (q + 1) * GRAD_SPLIT), 0, cur});
        }
    };
    std::vector<GradItem> it_a, it_b;
    std::vector<GradReduceItem> red_a, red_b;
    plan_items(want_b, b->d_out, it_b, red_b);
    plan_items(want_a, b->d_in, it_a, red_a);
    Blob blob;
    const size_t o_seg = blob.add(sd.data(), sd.size());
    const size_t o_off = blob.add(b->seg_offsets, (size_t)bi.S + 1);
    const size_t o_ita = blob.add(it_a.data(), it_a.size());
    const size_t o_itb = blob.add(it_b.data(), it_b.size());
    const size_t o_rda = blob.add(red_a.data(), red_a.size());
    const size_t o_rdb = blob.add(red_b.data(), red_b.size());
    const size_t o_chh = blob.add(ch_h.data(), ch_h.size());
    const size_t o_chd = blob.add(ch_dh.data(), ch_dh.size());
    const size_t o_pk = blob.add(pk_off.data(), pk_off.size());
    const size_t o_wl = blob.add(want_l.data(), want_l.size());
    const size_t o_wli = blob.add(want_lin.data(), want_lin.size());
    const size_t o_xs = blob.add(X_seg, seg_io ? (size_t)bi.S : 0);
    const size_t o_gs = blob.add(dY_seg, seg_io ? (size_t)bi.S : 0);
    const size_t o_ys = blob.add(Ybase_seg, (seg_io && Ybase_seg) ? (size_t)bi.S : 0);
    unsigned char* dev = nullptr;
    if ((st = upload(h, blob, s, &dev)) != SYMB_OK) return st;
    if ((st = fill_zeros()) != SYMB_OK) return st;
    unsigned char* wsb = (unsigned char*)ws;
    const SegDesc* dseg = (const SegDesc*)(dev + o_seg);
    const int32_t* doff = (const int32_t*)(dev + o_off);

    auto run_skinny_h = [&]() -> symb_status {          // Hs = s X A^T of the segments that want dB
        SkinnyParams sp{};
        sp.L = (const bf16*)X;
        sp.out = (bf16*)(wsb + wl.h_off);
        sp.K = b->d_in;
        sp.out_pitch = 2 * bi.max_rpad;
        sp.chunks = (const RowChunk*)(dev + o_chh);
        sp.seg = dseg;
        sp.use_packed = 0;
        if (seg_io) {
            sp.L_seg = (const bf16* const*)(dev + o_xs);
            sp.off = doff;
        }
        return launch_skinny(h, sp, (int)ch_h.size(), grad_max_rpad, s);
    };
    auto run_pack = [&]() -> symb_status {
        PackParams pp{dseg, (bf16*)(wsb + wl.pk_off), (const int64_t*)(dev + o_pk), b->d_out};
        hipLaunchKernelGGL(symb_pack_bt_kernel, dim3((b->d_out + 255) / 256, bi.S), dim3(256), 0, s, pp);
        SYMB_HIP(h, hipGetLastError());
        return SYMB_OK;
    };
    // One pass over dY for dB and dH: when both gradients are wanted of the same segments, dH has to be
    // computed here anyway, and the ranks fit one rank block.  The pass leaves dH in the workspace where an
    // input-gradient call with SYMB_BWD_REUSE_DH (same batch, same dY, same workspace) takes it.
    const bool one_pass = !reuse_dh && want_a == want_b && !want_b.empty() && bi.max_rpad == 16 && wl.dp_bytes;
    bool have_dh = reuse_dh;
    if (one_pass) {
        if (!reuse_hs && (st = run_skinny_h()) != SYMB_OK) return st;
        if ((st = run_pack()) != SYMB_OK) return st;
        DhDbParams dp{(const bf16*)dY, (const bf16*)(wsb + wl.h_off), (const bf16*)(wsb + wl.pk_off), (const int64_t*)(dev + o_pk),
                      b->d_out, 2 * bi.max_rpad, doff, dseg, (const GradItem*)(dev + o_itb), acc ? 1 : 0,
                      seg_io ? (const bf16* const*)(dev + o_gs) : nullptr, (float*)(wsb + wl.gr_off), (float*)(wsb + wl.dp_off), bi.T};
        const int groups = dhdb_groups(b->d_out);
        if (dhdb_blocks_per_group(b->d_out) == 2) hipLaunchKernelGGL(symb_lora_dhdb_kernel<2>, dim3(groups, (unsigned)it_b.size()), dim3(256), 0, s, dp);
        else hipLaunchKernelGGL(symb_lora_dhdb_kernel<4>, dim3(groups, (unsigned)it_b.size()), dim3(256), 0, s, dp);
        SYMB_HIP(h, hipGetLastError());
        if ((st = launch_grad_reduce(h, GradReduceParams{dseg, (const GradReduceItem*)(dev + o_rdb), (const float*)(wsb + wl.gr_off), b->d_out, 1, acc ? 1 : 0},
                                     (int)red_b.size(), s)) != SYMB_OK) return st;
        DhFinishParams fp{(const float*)(wsb + wl.dp_off), groups, bi.T, (bf16*)(wsb + wl.dh_off), 2 * bi.max_rpad,
                          (const RowChunk*)(dev + o_chd), dseg};
        hipLaunchKernelGGL(symb_dh_finish_kernel, dim3((unsigned)ch_dh.size()), dim3(128), 0, s, fp);
        SYMB_HIP(h, hipGetLastError());
        have_dh = true;
    } else if (!want_b.empty()) {       // dB_i = s_i * dY_i^T H_i  ==  dY_i^T Hs_i
        if (!reuse_hs && (st = run_skinny_h()) != SYMB_OK) return st;
        GradParams gp{(const bf16*)dY, (const bf16*)(wsb + wl.h_off), b->d_out, 2 * bi.max_rpad, doff, dseg,
                      (const GradItem*)(dev + o_itb), acc ? 1 : 0, seg_io ? (const bf16* const*)(dev + o_gs) : nullptr,
                      (float*)(wsb + wl.gr_off)};
        if ((st = launch_grad<true>(h, gp, (int)it_b.size(), grad_max_rpad, s)) != SYMB_OK) return st;
        if ((st = launch_grad_reduce(h, GradReduceParams{dseg, (const GradReduceItem*)(dev + o_rdb), (const float*)(wsb + wl.gr_off), b->d_out, 1, acc ? 1 : 0},
                                     (int)red_b.size(), s)) != SYMB_OK) return st;
    }
    if (!want_a.empty()) {       // dA_i = dH_i^T X_i
        if (!have_dh) {
            if ((st = run_pack()) != SYMB_OK) return st;
            SkinnyParams sp{};
            sp.L = (const bf16*)dY;
            sp.out = (bf16*)(wsb + wl.dh_off);
            sp.K = b->d_out;
            sp.out_pitch = 2 * bi.max_rpad;
            sp.chunks = (const RowChunk*)(dev + o_chd);
            sp.seg = dseg;
            sp.packed = (const bf16*)(wsb + wl.pk_off);
            sp.packed_off = (const int64_t*)(dev + o_pk);
            sp.use_packed = 1;
            if (seg_io) {
                sp.L_seg = (const bf16* const*)(dev + o_gs);
                sp.off = doff;
            }
            if ((st = launch_skinny(h, sp, (int)ch_dh.size(), grad_max_rpad, s)) != SYMB_OK) return st;
        }
        GradParams gp{(const bf16*)X, (const bf16*)(wsb + wl.dh_off), b->d_in, 2 * bi.max_rpad, doff, dseg,
                      (const GradItem*)(dev + o_ita), acc ? 1 : 0, seg_io ? (const bf16* const*)(dev + o_xs) : nullptr,
                      (float*)(wsb + wl.gr_off)};
        if ((st = launch_grad<false>(h, gp, (int)it_a.size(), grad_max_rpad, s)) != SYMB_OK) return st;
        if ((st = launch_grad_reduce(h, GradReduceParams{dseg, (const GradReduceItem*)(dev + o_rda), (const float*)(wsb + wl.gr_off), b->d_in, 0, acc ? 1 : 0},
                                     (int)red_a.size(), s)) != SYMB_OK) return st;
    }
    if (!want_l.empty()) {
        Ia3GradParams ip{(const bf16*)dY, (const bf16*)Ybase, b->d_out, doff, dseg, (const int32_t*)(dev + o_wl), acc ? 1 : 0,
                         seg_io ? (const bf16* const*)(dev + o_gs) : nullptr, seg_io ? (const bf16* const*)(dev + o_ys) : nullptr};
        hipLaunchKernelGGL(symb_ia3_grad_kernel, dim3((b->d_out + IA3_GRAD_COLS - 1) / IA3_GRAD_COLS, (unsigned)want_l.size()), dim3(256), 0, s, ip);
        SYMB_HIP(h, hipGetLastError());
    }
    if (!want_lin.empty()) {     // dl_i[k] = sum_t X[t][k] * (dY W)[t][k]: the same reduction over the input width
        Ia3GradParams ip{(const bf16*)X, (const bf16*)dXbase, b->d_in, doff, dseg, (const int32_t*)(dev + o_wli), acc ? 1 : 0,
                         seg_io ? (const bf16* const*)(dev + o_xs) : nullptr, seg_io ? (const bf16* const*)(dev + o_ys) : nullptr};
        hipLaunchKernelGGL(symb_ia3_grad_kernel, dim3((b->d_in + IA3_GRAD_COLS - 1) / IA3_GRAD_COLS, (unsigned)want_lin.size()), dim3(256), 0, s, ip);
        SYMB_HIP(h, hipGetLastError());
    }
    { guard.completed = true; return seal_slot(h, s); }
}

}  // extern "C"
