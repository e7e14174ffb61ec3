/* Plain C99 client of the library: proves that include/sentry.h is a C header and that the
 * shared library can be used without Python or C++.  Touches only host-side behaviour
 * (digest comparison, argument checks, error text), so it runs without a GPU. */
#include <stdio.h>
#include <string.h>

#include "sentry.h"

static int fails = 0;
#define EXPECT(cond)                                                     \
    do {                                                                 \
        if (!(cond)) { printf("FAIL line %d: %s\n", __LINE__, #cond); fails++; } \
    } while (0)

int main(void)
{
    uint8_t a[SENTRY_DIGEST_BYTES], b[SENTRY_DIGEST_BYTES];
    uint16_t lanes[SENTRY_LANES];
    const void *ptrs[1] = {(const void *)0x1000};
    size_t lens[1] = {64};
    int i;

    for (i = 0; i < SENTRY_DIGEST_BYTES; i++) a[i] = b[i] = (uint8_t)(3 * i + 1);
    EXPECT(sentry_verify(a, b) == SENTRY_OK);
    EXPECT(strcmp(sentry_last_error(), "") == 0);
    b[0] ^= 1;
    EXPECT(sentry_verify(a, b) == SENTRY_MISMATCH);
    b[0] ^= 1;
    b[SENTRY_DIGEST_BYTES - 1] ^= 0x80;
    EXPECT(sentry_verify(a, b) == SENTRY_MISMATCH);
    EXPECT(sentry_verify(NULL, b) == SENTRY_ERR_INVALID_ARG);
    EXPECT(strstr(sentry_last_error(), "NULL") != NULL);

    /* argument errors are found before any GPU work */
    EXPECT(sentry_merkle_root((const void *)0x1000, 4096, 100, a, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(strstr(sentry_last_error(), "leaf_bytes") != NULL);
    EXPECT(sentry_merkle_root((const void *)0x1004, 4096, 64, a, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_merkle_root_h(7, (const void *)0x1000, 4096, 64, a, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_merkle_segments(ptrs, lens, 0, 64, NULL, a, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_merkle_inplace_h(SENTRY_HASH_SHA3_256, ptrs, lens, 1, 64, NULL, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_lthash((const void *)0x1000, NULL, 5, lanes, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_lthash_model(ptrs, lens, 1, 100, NULL, lanes, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_lthash_combine(NULL, lanes, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_lthash32((const void *)0x1000, NULL, 5, lanes, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_lthash_fixed(NULL, 100, 5, lanes, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_merkle_coalesced(ptrs, lens, 1, 100, NULL, 0, a, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_reserve_scratch(1000, 100, 0, NULL) == SENTRY_ERR_INVALID_ARG);
    EXPECT(sentry_scratch_bytes(NULL, NULL, NULL) == SENTRY_ERR_INVALID_ARG);
    {   /* a host-only call with a result: one 64-byte tensor in 128-byte blocks is one gathered block */
        size_t gathered = 1, copied = 1, runs = 0;
        EXPECT(sentry_merkle_coalesced_plan(ptrs, lens, 1, 128, &gathered, &copied, &runs) == SENTRY_OK);
        EXPECT(gathered == 128 && copied == 64 && runs == 1);
        EXPECT(sentry_merkle_coalesced_plan(ptrs, lens, 1, 64, &gathered, &copied, &runs) == SENTRY_OK);
        EXPECT(gathered == 0 && copied == 0 && runs == 1);
    }
    /* a successful host-only call clears the text */
    EXPECT(sentry_verify(a, a) == SENTRY_OK);
    EXPECT(strcmp(sentry_last_error(), "") == 0);

    if (fails) return 1;
    printf("abi smoke ok\n");
    return 0;
}
