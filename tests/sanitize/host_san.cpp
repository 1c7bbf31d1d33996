// Runs the host-only parts of the library (argument checks, the segment planner, the row map, the
// workspace figures, the batching queue) so that a host build with -fsanitize=address,undefined can
// watch them.  No GPU call is made.  Prints one line; exit status 0 = every call returned what it should.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/symb.h"
#include "../../include/symb_batcher.h"

static unsigned lcg = 777u;
static unsigned rnd(unsigned n) {
    lcg = lcg * 1664525u + 1013904223u;
    return (lcg >> 8) % n;
}

int main() {
    int fails = 0;
    long sum = 0;
    alignas(16) static unsigned char fake[64];           // stands for device memory: never dereferenced by host-only calls
    for (int trial = 0; trial < 200; ++trial) {
        const int S = (int)rnd(40);
        std::vector<int32_t> off(S + 1, 0);
        std::vector<symb_adapter> ad(S);
        for (int i = 0; i < S; ++i) {
            const unsigned k = rnd(5);
            off[i + 1] = off[i] + (k == 0 ? 0 : k == 1 ? 1 : (int)rnd(700));
            ad[i] = symb_adapter{};
            ad[i].kind = (int32_t)rnd(4);
            if (ad[i].kind == SYMB_ADAPTER_LORA) {
                ad[i].rank = 1 + (int32_t)rnd(SYMB_MAX_RANK);
                ad[i].scale = 2.f;
                ad[i].A = fake;
                ad[i].B = fake;
                if (rnd(2)) { ad[i].dA = fake; ad[i].dB = fake; }
            } else if (ad[i].kind != SYMB_ADAPTER_NONE) {
                ad[i].A = fake;
            }
        }
        symb_batch b{};
        b.d_in = 8 * (1 + (int)rnd(600));
        b.d_out = 8 * (1 + (int)rnd(600));
        b.num_segments = S;
        b.seg_offsets = off.data();
        b.adapters = ad.data();
        b.weight_layout = (int32_t)rnd(2);
        fails += symb_validate_batch(&b) != SYMB_OK;
        const int T = off[S];
        std::vector<int32_t> map(T + 1, -1);
        fails += symb_debug_row_segment_map(&b, map.data()) != SYMB_OK;
        for (int t = 0; t < T; ++t) {
            fails += !(off[map[t]] <= t && t < off[map[t] + 1]);
            sum += map[t];
        }
        for (int tile : {32, 128, 256}) {
            const int nt = (T + tile - 1) / tile;
            std::vector<int32_t> lo(nt + 1, -7), hi(nt + 1, -7);
            int32_t n = -1;
            fails += symb_plan_row_tiles(&b, tile, lo.data(), hi.data(), &n) != SYMB_OK || n != nt;
            for (int u = 0; u < nt; ++u) {
                fails += !(off[lo[u]] <= u * tile && u * tile < off[lo[u] + 1]);
                const int last = (u + 1) * tile < T ? (u + 1) * tile - 1 : T - 1;
                fails += !(off[hi[u]] <= last && last < off[hi[u] + 1]);
                sum += lo[u] + hi[u];
            }
            fails += lo[nt] != -7 || hi[nt] != -7;               // nothing written past the tile count
        }
        for (int op = SYMB_OP_FWD; op <= SYMB_OP_BWD_INPUT_INPLACE; ++op) {
            size_t bytes = 0;
            fails += symb_workspace_bytes(&b, op, &bytes) != SYMB_OK;
            sum += (long)(bytes >> 8);
        }
        // bad batches are refused, with nothing read past the arrays
        if (S >= 2 && off[S] > off[S - 1]) {
            std::vector<int32_t> bad = off;
            bad[S] = bad[S - 1] - 1 < 0 ? -1 : bad[S - 1] - 1;
            if (bad[S] < bad[S - 1]) {
                symb_batch c = b;
                c.seg_offsets = bad.data();
                fails += symb_validate_batch(&c) != SYMB_ERR_BAD_SEGMENTS;
            }
        }
        symb_batch c = b;
        c.d_in = 12;
        fails += symb_validate_batch(&c) != SYMB_ERR_INVALID_ARG;
    }
    // the batching queue on a random arrival sequence, small take capacities included
    symb_batch_policy pol{50.0, 0.5, 800.0, 4096, 0};
    symb_batcher q = nullptr;
    fails += symb_batcher_create(&q, &pol, 3) != SYMB_OK;
    double now = 0.0;
    int64_t served = 0, submitted = 0;
    for (int i = 0; i < 2000; ++i) {
        now += rnd(400);
        symb_request r{};
        r.id = i;
        r.n_tokens = rnd(3) ? 1 + (int)rnd(4) : 64 + (int)rnd(5000);
        r.latency_sensitive = r.n_tokens < 8;
        r.arrival_us = now;
        const int layer = (int)rnd(3);
        fails += symb_batcher_submit(q, layer, &r) != SYMB_OK;
        ++submitted;
        for (int l = 0; l < 3; ++l) {
            const int cap = 1 + (int)rnd(6);
            std::vector<int64_t> ids(cap);
            std::vector<int32_t> so(cap + 1);
            int32_t n = -1;
            fails += symb_batcher_take(q, l, now, cap, ids.data(), so.data(), &n) != SYMB_OK || n < 0 || n > cap;
            served += n;
            for (int k = 0; k < n; ++k) sum += ids[k] + so[k + 1];
        }
    }
    for (int l = 0; l < 3; ++l)
        for (;;) {
            int64_t ids[8];
            int32_t so[9], n = 0;
            fails += symb_batcher_take(q, l, 1e18, 8, ids, so, &n) != SYMB_OK;
            if (n == 0) break;
            served += n;
        }
    fails += served != submitted;
    symb_request bad{};
    bad.n_tokens = 0;
    fails += symb_batcher_submit(q, 0, &bad) != SYMB_ERR_INVALID_ARG;
    fails += symb_batcher_submit(q, 9, &bad) != SYMB_ERR_INVALID_ARG;
    fails += symb_batcher_destroy(q) != SYMB_OK;
    std::printf("host_san fails=%d checksum=%ld\n", fails, sum);
    return fails ? 1 : 0;
}
