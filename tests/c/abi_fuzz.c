/* Host-side fuzz of the C ABI for a machine WITHOUT a GPU: with the pointer checks off every
 * call runs its whole planning arithmetic on random sizes, alignments and tunings and then
 * fails at the launch (no device), so only status codes come back.  Run against a library
 * whose host code is built with ASan + UBSan, any overflow or out-of-range shift aborts.
 * The buffers are made-up addresses: the program refuses to run where a device is usable. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include "brace.h"
#include "brace_tuning.h"

static uint64_t s = 0x9E3779B97F4A7C15ull;
static uint64_t rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }
static int64_t pick(const int64_t* v, int n) { return v[rnd() % n]; }

int main(void)
{
    static const int64_t ns[] = {1, 2, 3, 4, 7, 8, 15, 16, 47, 48, 100, 255, 256, 1000, 32767, 32768, 0, -1};
    static const int64_t ds[] = {0, 1, 31, 32, 33, 63, 64, 255, 256, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 65536,
                                 100003, 524288, 524289, 1000003, 11173962, 25000000, 100000000, 4000000000LL,
                                 (int64_t)1 << 40, (int64_t)1 << 45, ((int64_t)1 << 45) + 1, (int64_t)1 << 62, INT64_MAX, -1};
    static const int64_t pads[] = {0, 0, 1, 2, 3, 4, 8, 31, 32, 1000};
    static const float lams[] = {-1e30f, -40000.f, -1.f, 0.f, 0.5f, 5.f, 99.f, 100.f, 32767.f, 1e9f, 3e38f};
    const uintptr_t base_in = 0x7F0000000000ull, base_out = 0x7F8000000000ull, base_aux = 0x7FC000000000ull;
    long counts[4] = {0, 0, 0, 0};
    if (brace_init_device() == BRACE_OK) {
        printf("abi_fuzz: a GPU is usable here; refusing to launch on made-up addresses\n");
        return 77;
    }
    const int iterations = 200000;
    brace_set_pointer_checks(0);
    for (int it = 0; it < iterations; ++it) {
        const int64_t n = pick(ns, sizeof ns / sizeof *ns), d = pick(ds, sizeof ds / sizeof *ds);
        const int64_t pad = pick(pads, sizeof pads / sizeof *pads);
        brace_params_t p;
        brace_params_init(&p);
        p.lambda = lams[rnd() % (sizeof lams / sizeof *lams)];
        if (n > 0 && (rnd() % 3) == 0) {        /* the saturation corners of the threshold, relative to n */
            const float corners[] = {(float)n, (float)n - 0.5f, (float)n - 1.0f, -(float)n - 1.0f,
                                     -(float)n - 0.5f, -(float)n, -(float)n + 0.5f};
            p.lambda = corners[rnd() % (sizeof corners / sizeof *corners)];
        }
        p.zero_sign = (int)(rnd() % 3) - 1;
        p.rule = (rnd() % 8) == 0;
        p.ld = (rnd() % 3) ? 0 : (d >= 0 && d < INT64_MAX - 2000 ? d + pad : d);
        const float* in = (const float*)(base_in + 4 * (rnd() % 4));
        float* out = (rnd() % 5) ? (float*)(base_out + 4 * (rnd() % 5)) : NULL;
        p.out_bits_dev = (rnd() % 2) ? (void*)(base_aux + 4 * (rnd() % 2)) : NULL;
        p.sums_dev = (rnd() % 3) == 0 ? (int16_t*)(base_aux + 0x100000000ull + 2 * (rnd() % 4)) : NULL;
        brace_tuning_t t;
        brace_get_tuning(&t);
        t.vec = (int)(rnd() % 5); if (t.vec == 3) t.vec = 0;
        t.cols = (int[]){0, 0, 1, 2, 4, 8}[rnd() % 6];
        t.unroll = (int[]){0, 0, 2, 4, 8}[rnd() % 5];
        t.nontemporal = (int)(rnd() % 2); t.pipeline = (int)(rnd() % 2);
        t.split_writes = (int)(rnd() % 3); t.rowsplit = (int)(rnd() % 3); t.stage_writes = (int)(rnd() % 3);
        if (brace_set_tuning(&t) != BRACE_OK) { printf("tuning rejected\n"); return 1; }
        const int64_t f = n > 0 ? (int64_t)(rnd() % (uint64_t)(n + 1)) : 0;
        const int64_t c = n > 0 ? (int64_t)(rnd() % (uint64_t)(n + 2)) - 1 : 0;
        int rc;
        switch (rnd() % 15) {
        case 0: rc = brace_aggregate(in, n, d, f, &p, out, NULL); break;
        case 1: rc = brace_aggregate_chunk(in, n, d, f, c, &p, out, NULL); break;
        case 2: rc = brace_aggregate_chunks(in, n, d, f, c, c + (int64_t)(rnd() % 5), &p, out, NULL); break;
        case 3: rc = brace_aggregate_update(in, n, d, f, &p, 0.01f, out, NULL); break;
        case 4: rc = brace_aggregate_update_chunk(in, n, d, f, c, &p, 0.01f, out, NULL); break;
        case 5: { brace_rar_params_t rp = {sizeof(brace_rar_params_t), (int32_t)(rnd() % 2), p.ld,
                                           (int32_t)(rnd() % 2), 0};
                  rc = (rnd() % 2) ? brace_rar_aggregate(in, n, d, &rp, out, NULL)
                                   : brace_rar_aggregate_chunk(in, n, d, c, &rp, out, NULL); break; }
        case 6: rc = brace_quantize(in, n, d, p.ld, (uint32_t*)(base_aux + 16 * (rnd() % 2)),
                                    (rnd() % 3) == 0 ? 0 : (rnd() % 2) ? brace_packed_row_pitch(d)
                                    : brace_packed_row_words(d) + 4 * (int64_t)(rnd() % 3), NULL); break;
        case 7: p.sums_dev = NULL; p.rule = 0;
                rc = brace_vote_packed((const uint32_t*)base_in, n, d, 0, f, &p, out ? (float*)base_out : NULL, NULL); break;
        case 8: p.sums_dev = NULL; p.rule = 0;
                rc = brace_vote_packed_chunks((const uint32_t*)base_in, n, d, 0, f, c, c + (int64_t)(rnd() % 5), &p,
                                              out ? (float*)base_out : NULL, NULL); break;
        case 9: p.sums_dev = NULL; p.rule = 0;
                rc = brace_consensus_sums((const int16_t*)(base_in + 2 * (rnd() % 9)), n, d, p.ld, &p, out, NULL); break;
        case 12: rc = brace_quantize_1bit(in, n, d, p.ld, (int32_t)(rnd() % 4) - 1,
                                          (uint32_t*)(base_aux + 16 * (rnd() % 2)),
                                          (rnd() % 3) == 0 ? 0 : (rnd() % 2) ? brace_1bit_row_pitch(d)
                                          : brace_1bit_row_words(d) + 4 * (int64_t)(rnd() % 3), NULL); break;
        case 13: p.sums_dev = NULL; p.rule = 0;
                 rc = brace_vote_1bit((const uint32_t*)base_in, n, d, 0, f, &p, out ? (float*)base_out : NULL, NULL); break;
        case 14: p.sums_dev = NULL; p.rule = 0;
                 rc = brace_vote_1bit_chunks((const uint32_t*)base_in, n, d, 0, f, c, c + (int64_t)(rnd() % 5), &p,
                                             out ? (float*)base_out : NULL, NULL); break;
        case 10: rc = brace_expand_bits((const void*)base_aux, d, out, NULL); break;
        default: rc = brace_apply_bits((const void*)base_aux, d, 0.01f, out, NULL); break;
        }
        if (rc < 0 || rc > 3) { printf("unexpected status %d\n", rc); return 1; }
        counts[rc]++;
    }
    brace_set_tuning(NULL);
    printf("abi_fuzz ok: OK %ld EINVAL %ld ERANGE %ld EHIP %ld\n", counts[0], counts[1], counts[2], counts[3]);
    return 0;
}
