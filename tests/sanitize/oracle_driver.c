/* Sanitizer run of the CPU oracle (AddressSanitizer + UndefinedBehaviorSanitizer, host only):
 * key generation, encryption, every gate kind, a multiplexer and a small gate batch at a toy
 * parameter set, with the three product routines cross-checked.  Built and run by
 * tests/test_sanitizers.py; includes the oracle's source so that every static helper is
 * instrumented too. */
#include "../../oracle/tfhe_oracle.c"
#include <stdio.h>

int main(void)
{
    orc_params P = {16, 32, 1, 2, 10, 8, 2, -15, -25};
    if (orc_check_params(&P)) return 2;
    const int n = P.n, N = P.N;
    uint32_t *lwe = malloc(sizeof(uint32_t) * n), *ring = malloc(sizeof(uint32_t) * N);
    uint32_t *bk = malloc(sizeof(uint32_t) * orc_bk_words(&P)), *ksk = malloc(sizeof(uint32_t) * orc_ksk_words(&P));
    if (orc_keygen(&P, 99, lwe, ring, bk, ksk)) return 3;

    /* the three products agree */
    uint32_t a[32], b[32], c0[32], c1[32], c2[32];
    for (int j = 0; j < N; ++j) { a[j] = (uint32_t)orc_rand(1, 0, j); b[j] = (uint32_t)orc_rand(2, 0, j); }
    orc_negacyclic_definition(a, b, c0, N);
    orc_negacyclic_schoolbook(a, b, c1, N);
    orc_negacyclic_karatsuba(a, b, c2, N);
    if (memcmp(c0, c1, sizeof c0) || memcmp(c0, c2, sizeof c0)) return 4;

    /* truth tables of the six gates and of the multiplexer */
    const uint8_t bits[2] = {0, 1};
    uint32_t *ct = malloc(sizeof(uint32_t) * 2 * (n + 1)), *out = malloc(sizeof(uint32_t) * (n + 1));
    orc_encrypt(&P, lwe, 7, bits, 2, ct);
    static const int truth[6][4] = {{1, 1, 1, 0}, {0, 0, 0, 1}, {0, 1, 1, 1}, {1, 0, 0, 0}, {0, 1, 1, 0}, {1, 0, 0, 1}};
    for (int op = 0; op < 6; ++op)
        for (int x = 0; x < 2; ++x)
            for (int y = 0; y < 2; ++y) {
                uint8_t got;
                if (orc_gate(&P, bk, ksk, op, ct + x * (n + 1), 0, ct + y * (n + 1), 0, out)) return 5;
                orc_decrypt(&P, lwe, out, 1, &got);
                if (got != truth[op][2 * x + y]) return 6;
            }
    for (int s = 0; s < 2; ++s) {
        uint8_t got;
        if (orc_mux(&P, bk, ksk, ct + s * (n + 1), 0, ct + (n + 1), 0, ct, 1, out)) return 7;
        orc_decrypt(&P, lwe, out, 1, &got);      /* s ? 1 : NOT 0 */
        if (got != 1) return 8;
    }
    /* a batch with a multiplexer pair, two threads */
    uint32_t *wires = calloc((size_t)6 * (n + 1), sizeof(uint32_t));
    memcpy(wires, ct, sizeof(uint32_t) * 2 * (n + 1));
    orc_gate_rec g[4] = {{OP_XOR, 0, 1, 0, 0, 1, 2}, {OP_MUX, 0, 0, 0, 1, 0, 3}, {OP_MUX_ELSE, 0, 1, 0, 1, 0, 3},
                         {OP_NAND, 1, 0, 0, 0, 1, 4}};
    if (orc_gate_batch(&P, bk, ksk, g, 4, wires, 2)) return 9;
    uint8_t res[3];
    orc_decrypt(&P, lwe, wires + 2 * (size_t)(n + 1), 3, res);
    /* 0 XOR NOT 1 = 0;  1 ? 0 : NOT 0 = 0;  NAND(NOT 0, 1) = 0 */
    if (res[0] != 0 || res[1] != 0 || res[2] != 0) return 10;
    free(lwe); free(ring); free(bk); free(ksk); free(ct); free(out); free(wires);
    puts("oracle sanitizer run: ok");
    return 0;
}
