/* Host-side check of libfd's C ABI, meant to be built and run with AddressSanitizer and
 * UndefinedBehaviorSanitizer (host code only; no kernel is launched): every entry point with
 * arguments that must be refused before any device work, the workspace formula, the
 * thread-local error text.  Exit status 0 = every check held. */
#include <pthread.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fd.h"

static int failures = 0;
#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            ++failures;                                                              \
            fprintf(stderr, "FAILED line %d: %s   (last error: %s)\n", __LINE__, #cond, fd_last_error()); \
        }                                                                            \
    } while (0)

static fd_config good(void)
{
    fd_config c;
    memset(&c, 0, sizeof c);
    c.B = 2; c.Hq = 8; c.Hkv = 2; c.D = 128; c.S_max = 4096; c.max_splits = 16;
    return c;
}

static void* other_thread(void* arg)
{
    (void)arg;
    CHECK(strcmp(fd_last_error(), "") == 0);          /* this thread has made no failing call yet */
    fd_config c = good();
    c.D = 64;
    fd_handle_t h = (fd_handle_t)0x1;
    CHECK(fd_create(&c, &h) == FD_ERR_UNSUPPORTED && h == NULL);
    CHECK(strstr(fd_last_error(), "D = 128") != NULL);
    return NULL;
}

int main(void)
{
    CHECK(fd_version() == FD_VERSION);
    CHECK(strcmp(fd_last_error(), "") == 0);

    /* workspace formula: partials, one 128-byte line of LSEs per slot; second-level partials (one group of 16
     * splits here) and their LSE lines; tile counters, 64 group counters per tile, direct marks and the status
     * word, each array rounded up to 256 bytes */
    fd_config c = good();
    const size_t tiles = 4, G = 4, n = 16, groups = 1;
    CHECK(fd_workspace_bytes(&c) == tiles * n * G * 128 * 4 + tiles * n * 128 + tiles * groups * G * 128 * 4 +
                                        tiles * groups * 128 + 256 + tiles * 64 * 4 + 256 + 256);
    CHECK(fd_workspace_bytes(NULL) == 0);

    /* configurations that must be refused, by fd_workspace_bytes, fd_create and fd_decode_static alike */
    struct { fd_config c; int code; } bad[12];
    int nb = 0;
#define BAD(field, value, err) do { bad[nb].c = good(); bad[nb].c.field = (value); bad[nb].code = (err); ++nb; } while (0)
    BAD(B, 0, FD_ERR_INVALID_ARG);
    BAD(Hq, 7, FD_ERR_INVALID_ARG);
    BAD(S_max, -5, FD_ERR_INVALID_ARG);
    BAD(max_splits, 0, FD_ERR_INVALID_ARG);
    BAD(max_splits, FD_MAX_SPLITS + 1, FD_ERR_INVALID_ARG);
    BAD(scale, -1.0f, FD_ERR_INVALID_ARG);
    BAD(k_scale, -2.0f, FD_ERR_INVALID_ARG);
    BAD(D, 64, FD_ERR_UNSUPPORTED);
    BAD(kv_layout, 1, FD_ERR_UNSUPPORTED);
    BAD(dtype, 3, FD_ERR_UNSUPPORTED);
    BAD(Hq, 2 * 17, FD_ERR_UNSUPPORTED);               /* group of 17 */
    for (int i = 0; i < nb; ++i) {
        fd_handle_t h = (fd_handle_t)0x1;
        CHECK(fd_workspace_bytes(&bad[i].c) == 0);
        CHECK(fd_create(&bad[i].c, &h) == bad[i].code && h == NULL);
        CHECK(strlen(fd_last_error()) > 0);
        CHECK(fd_decode_static(&bad[i].c, NULL, NULL, NULL, NULL, NULL, NULL, 1, NULL) == bad[i].code);
    }
    CHECK(fd_create(&c, NULL) == FD_ERR_INVALID_ARG);
    {
        fd_handle_t h = (fd_handle_t)0x1;
        CHECK(fd_create(NULL, &h) == FD_ERR_INVALID_ARG && h == NULL);
    }

    /* a shape beyond the static workspace is refused before any device call */
    {
        fd_config big = good();
        big.B = 64; big.Hq = 32; big.Hkv = 8; big.S_max = 1024; big.max_splits = 64;
        CHECK(fd_workspace_bytes(&big) > FD_STATIC_SCRATCH_BYTES);
        CHECK(fd_decode_static(&big, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) == FD_ERR_WORKSPACE);
        CHECK(strstr(fd_last_error(), "static workspace") != NULL);
    }

    /* not a handle: NULL, and memory that does not carry the handle's mark */
    void* fake = calloc(1, 4096);
    fd_handle_t hs[2] = {NULL, (fd_handle_t)fake};
    for (int i = 0; i < 2; ++i) {
        fd_handle_t h = hs[i];
        int32_t v = 0;
        uint32_t counters[4];
        float us = 0.f;
        CHECK(fd_destroy(h) == FD_ERR_INVALID_ARG);
        CHECK(fd_reset(h, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_decode(h, fake, fake, fake, (const int32_t*)fake, (float*)fake, NULL, 1, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_decode_bsp(h, fake, fake, fake, (const int32_t*)fake, (float*)fake, NULL, 1, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_decode_waits(h, fake, fake, fake, (const int32_t*)fake, (float*)fake, NULL, 1, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_decode_paged(h, fake, fake, fake, (const int32_t*)fake, 16, 4, 4, (const int32_t*)fake, (float*)fake, NULL, 1, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_decode_paged_bsp(h, fake, fake, fake, NULL, 16, 4, 4, (const int32_t*)fake, (float*)fake, NULL, 1, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_autotune(h, fake, fake, fake, (const int32_t*)fake, (float*)fake, NULL, 1, NULL, 5, &us) == FD_ERR_INVALID_ARG);
        CHECK(fd_set_option(h, FD_OPT_PATH, 1) == FD_ERR_INVALID_ARG);
        CHECK(fd_get_option(h, FD_OPT_PATH, &v) == FD_ERR_INVALID_ARG);
        CHECK(fd_debug_poison_workspace(h, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_debug_read_counters(h, counters, 4) == FD_ERR_INVALID_ARG);
        CHECK(fd_debug_set_trace(h, NULL, 0) == FD_ERR_INVALID_ARG);
        CHECK(strstr(fd_last_error(), "handle") != NULL);
    }
    free(fake);
    {
        uint32_t sink = 0;
        CHECK(fd_debug_stream_read(NULL, 1024, &sink, NULL) == FD_ERR_INVALID_ARG);
        CHECK(fd_debug_stream_read(&sink, 8, &sink, NULL) == FD_ERR_INVALID_ARG);
    }

    /* a valid configuration: succeeds on a gfx950 device, fails cleanly anywhere else; either way nothing leaks */
    {
        fd_handle_t h = NULL;
        const int rc = fd_create(&c, &h);
        if (rc == FD_OK) {
            int32_t v = -1;
            CHECK(h != NULL);
            CHECK(fd_set_option(h, FD_OPT_XCD_GROUPS, 4) == FD_ERR_INVALID_ARG);
            CHECK(fd_set_option(h, FD_OPT_SPLIT_KEYS, 100) == FD_ERR_INVALID_ARG);
            CHECK(fd_set_option(h, FD_OPT_SPLIT_KEYS, 256) == FD_OK && fd_get_option(h, FD_OPT_SPLIT_KEYS, &v) == FD_OK && v == 256);
            CHECK(fd_get_option(h, FD_OPT_PATH, NULL) == FD_ERR_INVALID_ARG);
            CHECK(fd_decode(h, NULL, NULL, NULL, NULL, NULL, NULL, 1, NULL) == FD_ERR_INVALID_ARG);
            CHECK(fd_destroy(h) == FD_OK);
        } else {
            CHECK(h == NULL && (rc == FD_ERR_HIP || rc == FD_ERR_UNSUPPORTED || rc == FD_ERR_WORKSPACE));
            CHECK(strlen(fd_last_error()) > 0);
        }
    }

    /* the error text belongs to the calling thread */
    {
        fd_config b2 = good();
        b2.B = 0;
        fd_handle_t h = NULL;
        CHECK(fd_create(&b2, &h) == FD_ERR_INVALID_ARG);
        pthread_t t;
        CHECK(pthread_create(&t, NULL, other_thread, NULL) == 0);
        pthread_join(t, NULL);
        CHECK(strstr(fd_last_error(), "positive") != NULL);    /* untouched by the other thread's error */
    }

    printf("%s (%d failed checks)\n", failures ? "FAIL" : "OK", failures);
    return failures ? 1 : 0;
}
