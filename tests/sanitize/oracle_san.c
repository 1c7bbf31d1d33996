/* Runs every entry point of the CPU oracle on a small ragged batch (an empty segment, every adapter
 * kind, sampled rows and columns, per-token and broadcast noise, bad arguments) so that a build
 * with -fsanitize=address,undefined can watch all of its indexing.  Prints one checksum line;
 * exit status 0 = every call returned what it should. */
#include <stdio.h>
#include "../../oracle/symb_oracle.c"

static uint32_t lcg = 12345u;
static uint16_t rnd_bf16(void) {                      /* small values, sign and magnitude varied */
    lcg = lcg * 1664525u + 1013904223u;
    float f = ((int)((lcg >> 8) % 65) - 32) / 16.0f;
    union { float f; uint32_t u; } v;
    v.f = f;
    return (uint16_t)(v.u >> 16);
}
static void* owned[64];                               /* everything the driver allocates, freed before exit: */
static int n_owned = 0;                               /* what the leak check then reports is the oracle's */
static void* take(size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);
    owned[n_owned++] = p;
    return p;
}
static uint16_t* fill(size_t n) {
    uint16_t* p = (uint16_t*)take(sizeof(uint16_t) * n);
    for (size_t i = 0; i < n; ++i) p[i] = rnd_bf16();
    return p;
}

int main(void) {
    enum { D_IN = 24, D_OUT = 40, S = 5 };
    const int32_t off[S + 1] = {0, 7, 7, 8, 21, 30};   /* segment 1 is empty, segment 2 has one token */
    const int32_t T = off[S];
    uint16_t *X = fill((size_t)T * D_IN), *W = fill((size_t)D_OUT * D_IN), *bias = fill(D_OUT), *dY = fill((size_t)T * D_OUT);
    orc_adapter ad[S];
    memset(ad, 0, sizeof ad);
    ad[0].kind = ORC_LORA; ad[0].rank = 3; ad[0].scale = 2.0; ad[0].A = fill(3 * D_IN); ad[0].B = fill(D_OUT * 3);
    ad[1].kind = ORC_LORA; ad[1].rank = 5; ad[1].scale = 0.5; ad[1].A = fill(5 * D_IN); ad[1].B = fill(D_OUT * 5);
    ad[2].kind = ORC_IA3; ad[2].A = fill(D_OUT);
    ad[3].kind = ORC_IA3_IN; ad[3].A = fill(D_IN);
    ad[4].kind = ORC_NONE;
    double sum = 0.0;
    int fails = 0;
    /* all rows, then a sample with the first and the last row of the batch */
    double *Y0 = (double*)take(sizeof(double) * T * D_OUT), *Y = (double*)take(sizeof(double) * T * D_OUT);
    fails += orc_forward_rows(D_IN, D_OUT, S, off, ad, X, W, bias, T, NULL, Y0, Y) != 0;
    for (int i = 0; i < T * D_OUT; ++i) sum += Y[i] + 0.5 * Y0[i];
    const int32_t rows[4] = {0, 7, 20, T - 1};
    fails += orc_forward_rows(D_IN, D_OUT, S, off, ad, X, W, NULL, 4, rows, Y0, Y) != 0;
    for (int i = 0; i < 4 * D_OUT; ++i) sum += Y[i];
    const int32_t bad_rows[2] = {3, T};                /* a row past the batch must be reported, not read */
    fails += orc_forward_rows(D_IN, D_OUT, S, off, ad, X, W, NULL, 2, bad_rows, Y0, Y) == 0;
    double* dX = (double*)take(sizeof(double) * T * D_IN);
    for (int base_only = 0; base_only < 2; ++base_only) {
        fails += orc_backward_input_rows(D_IN, D_OUT, S, off, ad, dY, W, T, NULL, base_only, dX) != 0;
        for (int i = 0; i < T * D_IN; ++i) sum += dX[i];
    }
    fails += orc_backward_input_rows(D_IN, D_OUT, S, off, ad, dY, W, 4, rows, 0, dX) != 0;
    fails += orc_backward_input_rows(D_IN, D_OUT, S, off, ad, dY, W, 2, bad_rows, 0, dX) == 0;
    /* parameter gradients: a LoRA segment, the empty LoRA segment, both IA3 kinds with and without saved tensors */
    double *dA = (double*)take(sizeof(double) * 5 * D_IN), *dB = (double*)take(sizeof(double) * D_OUT * 5);
    fails += orc_lora_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, 0, dA, dB) != 0;
    for (int i = 0; i < 3 * D_IN; ++i) sum += dA[i];
    for (int i = 0; i < D_OUT * 3; ++i) sum += dB[i];
    fails += orc_lora_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, 1, dA, NULL) != 0;
    for (int i = 0; i < 5 * D_IN; ++i) fails += dA[i] != 0.0;
    fails += orc_lora_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, 2, dA, dB) == 0;      /* not a LoRA segment */
    double* dl = (double*)take(sizeof(double) * D_OUT);
    uint16_t *Y0s = fill((size_t)T * D_OUT), *Gs = fill((size_t)T * D_IN);
    const int32_t cols[3] = {0, 5, D_IN - 1};
    fails += orc_ia3_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, W, bias, NULL, 2, D_OUT, NULL, dl, NULL) != 0;
    for (int i = 0; i < D_OUT; ++i) sum += dl[i];
    fails += orc_ia3_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, W, bias, Y0s, 2, 3, cols, dl, NULL) != 0;
    fails += orc_ia3_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, W, NULL, NULL, 3, D_IN, NULL, dl, NULL) != 0;
    for (int i = 0; i < D_IN; ++i) sum += dl[i];
    fails += orc_ia3_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, W, NULL, NULL, 3, 3, cols, dl, Gs) != 0;
    fails += orc_ia3_grad_segment(D_IN, D_OUT, S, off, ad, X, dY, W, NULL, NULL, 4, 3, cols, dl, NULL) == 0;   /* kind NONE */
    /* privacy flow: per-token noise, a broadcast row, none */
    const uint16_t* noise[S] = {fill(7 * D_IN), NULL, fill(D_IN), NULL, fill(D_IN)};
    const int32_t nrows[S] = {7, 0, 1, 0, 1};
    uint16_t* Xn = (uint16_t*)take(sizeof(uint16_t) * T * D_IN);
    fails += orc_noise_add(D_IN, S, off, X, noise, nrows, Xn) != 0;
    for (int i = 0; i < T * D_IN; ++i) sum += Xn[i] * 1e-6;
    fails += orc_forward_private_rows(D_IN, D_OUT, S, off, ad, Xn, W, bias, noise, nrows, T, NULL, Y) != 0;
    fails += orc_forward_private_rows(D_IN, D_OUT, S, off, ad, Xn, W, bias, noise, nrows, 4, rows, Y) != 0;
    for (int i = 0; i < 4 * D_OUT; ++i) sum += Y[i];
    const int32_t bad_n[S] = {3, 0, 1, 0, 1};          /* neither 1 nor the segment's length */
    fails += orc_noise_add(D_IN, S, off, X, noise, bad_n, Xn) == 0;
    /* the integer map and offset checks */
    int32_t* map = (int32_t*)take(sizeof(int32_t) * T);
    fails += orc_row_segment_map(S, off, map) != 0;
    for (int i = 0; i < T; ++i) sum += map[i];
    const int32_t bad_off[3] = {0, 5, 4};
    fails += orc_row_segment_map(2, bad_off, map) == 0;
    while (n_owned) free(owned[--n_owned]);
    printf("oracle_san fails=%d checksum=%.9e threads=%d\n", fails, sum, orc_num_threads());
    return fails ? 1 : 0;
}
