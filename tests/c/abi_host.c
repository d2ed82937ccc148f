/* The C ABI from plain C99: the header must compile as C, and the host-only entry points
 * and the argument validation must behave as documented without any GPU call being made.
 * Built and run by tests/test_abi_host.py. */
#include <math.h>
#include <stdio.h>
#include <string.h>

#include "brace.h"
#include "brace_tuning.h"

#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            printf("FAIL line %d: %s\n", __LINE__, #cond);               \
            return 1;                                                    \
        }                                                                \
    } while (0)

int main(void)
{
    brace_params_t p;
    int64_t lo = -1, hi = -1, owner = -1;
    const float* fake_in = (const float*)(uintptr_t)0x7f0000000000ull;   /* never dereferenced */
    float* fake_out = (float*)(uintptr_t)0x7f8000000000ull;

    brace_params_init(&p);
    CHECK(p.struct_size == sizeof(brace_params_t));
    CHECK(p.lambda == 5.0f && p.zero_sign == 0 && p.rule == 0 && p.ld == 0);
    CHECK(p.out_bits_dev == NULL && p.sums_dev == NULL);

    /* 1,000,003 coordinates over 20 clients: 3 chunks of 50,001, then 17 of 50,000 */
    CHECK(brace_chunk_range(20, 1000003, 0, &lo, &hi) == BRACE_OK && lo == 0 && hi == 50001);
    CHECK(brace_chunk_range(20, 1000003, 3, &lo, &hi) == BRACE_OK && lo == 150003 && hi == 200003);
    CHECK(brace_chunk_range(20, 1000003, 19, &lo, &hi) == BRACE_OK && hi == 1000003);
    CHECK(brace_chunk_range(20, 1000003, 20, &lo, &hi) == BRACE_ERANGE);
    CHECK(strlen(brace_last_error()) > 0);
    /* three-client ring: the second sub-vector ends on Client 1 */
    CHECK(brace_chunk_owner(3, 1, &owner) == BRACE_OK && owner == 0);
    CHECK(brace_chunk_owner(3, 0, &owner) == BRACE_OK && owner == 2);
    CHECK(brace_packed_row_words(25000000) == 2 * 781250);
    CHECK(brace_packed_row_words(33) == 4);
    /* recommended pitches: whole 128-byte lines per row */
    CHECK(brace_packed_row_pitch(25000000) == 1562528 && brace_packed_row_pitch(33) == 32);
    CHECK(brace_packed_row_pitch(0) == 0 && brace_packed_row_pitch(1024) == 64);
    CHECK(brace_1bit_row_words(25000000) == 781252 && brace_1bit_row_pitch(25000000) == 781280);
    CHECK(brace_1bit_row_pitch(1) == 32 && brace_1bit_row_pitch(1024) == 32 && brace_1bit_row_pitch(1025) == 64);

    /* Eq. (1) on integers: S > lambda <=> S >= T, saturating one step outside [-n, n] */
    {
        int32_t T = 0;
        CHECK(brace_threshold(100, 5.0f, &T) == BRACE_OK && T == 6);
        CHECK(brace_threshold(100, 4.999f, &T) == BRACE_OK && T == 5);
        CHECK(brace_threshold(100, -0.5f, &T) == BRACE_OK && T == 0);
        CHECK(brace_threshold(100, 99.5f, &T) == BRACE_OK && T == 100);
        CHECK(brace_threshold(100, 100.0f, &T) == BRACE_OK && T == 101);      /* lambda = n: all -1 */
        CHECK(brace_threshold(100, 1e30f, &T) == BRACE_OK && T == 101);
        CHECK(brace_threshold(100, -100.0f, &T) == BRACE_OK && T == -99);
        CHECK(brace_threshold(100, -100.5f, &T) == BRACE_OK && T == -100);
        CHECK(brace_threshold(100, -101.0f, &T) == BRACE_OK && T == -100);    /* lambda = -n-1: all +1 */
        CHECK(brace_threshold(100, -1e30f, &T) == BRACE_OK && T == -100);
        CHECK(brace_threshold(1, 0.0f, &T) == BRACE_OK && T == 1);
        CHECK(brace_threshold(BRACE_MAX_CLIENTS, 3e38f, &T) == BRACE_OK && T == BRACE_MAX_CLIENTS + 1);
        CHECK(brace_threshold(100, NAN, &T) == BRACE_EINVAL);
        CHECK(brace_threshold(0, 1.0f, &T) == BRACE_EINVAL);
        CHECK(brace_threshold(100, 1.0f, NULL) == BRACE_EINVAL);
    }

    CHECK(brace_aggregate(fake_in, 4, 100, 1, NULL, fake_out, NULL) == BRACE_EINVAL);
    CHECK(brace_aggregate(NULL, 4, 100, 1, &p, fake_out, NULL) == BRACE_EINVAL);
    CHECK(brace_aggregate(fake_in, 4, 100, 5, &p, fake_out, NULL) == BRACE_EINVAL);
    CHECK(brace_aggregate(fake_in, BRACE_MAX_CLIENTS + 1, 100, 0, &p, fake_out, NULL) == BRACE_ERANGE);
    p.lambda = NAN;
    CHECK(brace_aggregate(fake_in, 4, 100, 1, &p, fake_out, NULL) == BRACE_EINVAL);
    p.lambda = 5.0f;
    CHECK(brace_aggregate(fake_in, 4, 0, 1, &p, fake_out, NULL) == BRACE_OK);        /* d = 0 */
    CHECK(brace_aggregate_chunk(fake_in, 7, 3, 0, 6, &p, fake_out, NULL) == BRACE_OK); /* empty chunk */
    CHECK(brace_aggregate_chunks(fake_in, 4, 100, 1, 2, 2, &p, fake_out, NULL) == BRACE_OK);
    CHECK(brace_aggregate_update(fake_in, 4, 100, 1, &p, INFINITY, fake_out, NULL) == BRACE_EINVAL);
    CHECK(brace_expand_bits(NULL, 0, NULL, NULL) == BRACE_OK);
    /* buffers of one call must be pairwise disjoint: bits inside out, sums inside the matrix */
    p.out_bits_dev = (void*)(fake_out + 8);
    CHECK(brace_aggregate(fake_in, 4, 100, 1, &p, fake_out, NULL) == BRACE_EINVAL);
    CHECK(strstr(brace_last_error(), "overlaps") != NULL);
    p.out_bits_dev = NULL;
    p.sums_dev = (int16_t*)(uintptr_t)(0x7f0000000000ull + 64);
    CHECK(brace_aggregate(fake_in, 4, 100, 1, &p, fake_out, NULL) == BRACE_EINVAL);
    p.sums_dev = NULL;

    {
        brace_rar_params_t r;
        brace_rar_params_init(&r);
        CHECK(r.struct_size == sizeof(r) && r.mean == 0 && r.ld == 0 && r.order == 0 && r.reserved == 0);
        r.mean = 2;
        CHECK(brace_rar_aggregate(fake_in, 4, 100, &r, fake_out, NULL) == BRACE_EINVAL);
        r.mean = 1;
        CHECK(brace_rar_aggregate(fake_in, 4, 0, &r, fake_out, NULL) == BRACE_OK);
        r.order = 2;
        CHECK(brace_rar_aggregate(fake_in, 4, 100, &r, fake_out, NULL) == BRACE_EINVAL);
        r.order = 1;
        CHECK(brace_rar_aggregate(fake_in, 4, 0, &r, fake_out, NULL) == BRACE_OK);
        CHECK(brace_rar_aggregate_chunk(fake_in, 4, 100, 4, &r, fake_out, NULL) == BRACE_ERANGE);
        /* out inside the matrix: rejected before anything is launched */
        CHECK(brace_rar_aggregate(fake_in, 4, 100, &r, (float*)(uintptr_t)(0x7f0000000000ull + 40), NULL)
              == BRACE_EINVAL);
    }
    {
        brace_tuning_t t;
        CHECK(brace_get_tuning(&t) == BRACE_OK && t.struct_size == sizeof(t));
        t.cols = 3;
        CHECK(brace_set_tuning(&t) == BRACE_EINVAL);
        CHECK(brace_set_tuning(NULL) == BRACE_OK);
    }
    printf("abi_host ok\n");
    return 0;
}
