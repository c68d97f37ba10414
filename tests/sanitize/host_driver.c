/* Drives the host side of libhola's entry points (argument checks, workspace sizing, tuning, the timing aid's
 * bookkeeping) on a machine without a GPU; built with the library's sources under AddressSanitizer +
 * UndefinedBehaviorSanitizer (host code only) by tests/test_sanitizers.py.  Device pointers are fake and must never
 * be touched on the host.  A call whose arguments are valid goes on to the HIP runtime, which has no device here:
 * HOLA_ERR_HIP is then the expected answer (HOLA_OK where a GPU is present). */
#include <math.h>
#include <stdio.h>
#include <string.h>
#include "hola.h"

static int failures = 0;
#define EXPECT(call, want) do { hola_status got_ = (call); if (got_ != (want)) { ++failures; \
    printf("line %d: %s -> %d (%s), expected %d\n", __LINE__, #call, (int)got_, hola_status_string(got_), (int)(want)); } } while (0)
#define EXPECT_RAN(call) do { hola_status got_ = (call); if (got_ != HOLA_OK && got_ != HOLA_ERR_HIP) { ++failures; \
    printf("line %d: %s -> %d (%s), expected OK or HIP error\n", __LINE__, #call, (int)got_, hola_status_string(got_)); } } while (0)
#define CHECK(cond) do { if (!(cond)) { ++failures; printf("line %d: %s is false\n", __LINE__, #cond); } } while (0)

static void* const FAKE = (void*)0x1000;
static void* const WS = (void*)0x10000;

static hola_verify_args base_args(void)
{
    hola_verify_args a;
    memset(&a, 0, sizeof a);
    a.target_logits = FAKE; a.draft_logits = FAKE; a.draft_tokens = (const int32_t*)FAKE;
    a.out_accept_len = (int32_t*)FAKE; a.out_next_token = (int32_t*)FAKE;
    a.dtype = HOLA_DTYPE_BF16; a.B = 4; a.gamma = 3; a.V = 100;
    a.temperature = 1.0f; a.entropy_threshold = 2.0f;
    a.workspace = WS; a.workspace_bytes = (size_t)1 << 30;
    return a;
}

static hola_tree_args base_tree(void)
{
    hola_tree_args a;
    memset(&a, 0, sizeof a);
    a.target_logits = FAKE; a.draft_logits = FAKE; a.node_token = (const int32_t*)FAKE; a.node_parent = (const int32_t*)FAKE;
    a.out_accept_len = (int32_t*)FAKE; a.out_next_token = (int32_t*)FAKE;
    a.dtype = HOLA_DTYPE_BF16; a.B = 4; a.N = 6; a.V = 100;
    a.temperature = 1.0f; a.entropy_threshold = 2.0f;
    a.workspace = WS; a.workspace_bytes = (size_t)1 << 30;
    return a;
}

int main(void)
{
    printf("%s\n", hola_version());
    for (int st = HOLA_OK; st <= HOLA_ERR_HIP; ++st) CHECK(hola_status_string((hola_status)st) != NULL);
    CHECK(hola_last_hip_error() != NULL);

    /* ---- workspace sizes */
    CHECK(hola_workspace_bytes(0, 1, 1) > 0);
    CHECK(hola_workspace_bytes(-1, 8, 100) == 0 && hola_workspace_bytes(4, 0, 100) == 0 && hola_workspace_bytes(4, 64, 100) == 0 &&
          hola_workspace_bytes(4, 8, 0) == 0);
    CHECK(hola_workspace_bytes(256, 8, 128256) > hola_workspace_bytes(64, 8, 128256));
    CHECK(hola_workspace_bytes(1 << 20, 63, 1 << 30) > 0);          /* huge shapes: no overflow trap in the size arithmetic */
    {
        hola_verify_args a = base_args();
        a.B = 256; a.gamma = 8; a.V = 128256;
        const size_t plain = hola_workspace_bytes_ex(&a);
        a.top_k = 50;
        const size_t filt = hola_workspace_bytes_ex(&a);
        CHECK(plain > 0 && plain < filt && filt <= hola_workspace_bytes(256, 8, 128256));
        CHECK(plain <= (size_t)HOLA_STATIC_SCRATCH_BYTES);
        CHECK(hola_workspace_bytes_ex(NULL) == 0);
        a.gamma = 0;
        CHECK(hola_workspace_bytes_ex(&a) == 0);
    }
    CHECK(hola_hsd_workspace_bytes(1, 4, 2, 10) == 0 && hola_hsd_workspace_bytes(3, 4, 63, 10) == 0);
    CHECK(hola_hsd_workspace_bytes(3, 4, 2, 10) > hola_workspace_bytes(4, 3, 10));
    CHECK(hola_tree_workspace_bytes(4, 0, 100) == 0 && hola_tree_workspace_bytes(4, 64, 100) == 0 && hola_tree_workspace_bytes(4, 63, 100) > 0);
    CHECK(hola_tile_stats_workspace_bytes(4, 100, 0) == 0 && hola_tile_stats_workspace_bytes(4, 100, 32) > 0 &&
          hola_tile_stats_workspace_bytes(0, 100, 32) > 0);

    /* ---- one verify level: every refusal, then calls that reach the launches */
    EXPECT(hola_verify_ex(NULL), HOLA_ERR_INVALID_ARG);
    EXPECT(hola_verify_ex_static(NULL), HOLA_ERR_INVALID_ARG);
    { hola_verify_args a = base_args(); a.B = -1; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.gamma = 0; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.gamma = 64; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.V = 0; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.dtype = 7; EXPECT(hola_verify_ex(&a), HOLA_ERR_UNSUPPORTED); }
    { hola_verify_args a = base_args(); a.target_logits = NULL; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.draft_tokens = NULL; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.out_next_token = NULL; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.target_logits = (void*)0x1001; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.target_ld = 99; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.entropy_ld = 2; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.temperature = NAN; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.temperature = INFINITY; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.entropy_threshold = NAN; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.workspace = NULL; EXPECT(hola_verify_ex(&a), HOLA_ERR_WORKSPACE); }
    { hola_verify_args a = base_args(); a.workspace = (void*)0x10010; EXPECT(hola_verify_ex(&a), HOLA_ERR_WORKSPACE); }
    { hola_verify_args a = base_args(); a.workspace_bytes = 1024; EXPECT(hola_verify_ex(&a), HOLA_ERR_WORKSPACE); }
    { hola_verify_args a = base_args(); a.top_k = -3; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.top_p = -0.5f; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG); }
    { hola_verify_args a = base_args(); a.top_k = 5; a.temperature = 0.f; EXPECT(hola_verify_ex(&a), HOLA_ERR_UNSUPPORTED); }
    { hola_verify_args a = base_args(); a.top_k = 5; a.row_temperature = (const float*)FAKE; EXPECT(hola_verify_ex(&a), HOLA_ERR_UNSUPPORTED); }
    { hola_verify_args a = base_args(); a.target_stats_in = (const double*)FAKE; a.temperature = 0.f; EXPECT(hola_verify_ex(&a), HOLA_ERR_UNSUPPORTED); }
    { hola_verify_args a = base_args(); a.B = 0; EXPECT(hola_verify_ex(&a), HOLA_OK); EXPECT(hola_verify_ex_static(&a), HOLA_OK); }
    {   /* a tuning that is out of range is refused with the call; a valid one is taken */
        hola_tuning t; memset(&t, 0, sizeof t);
        hola_verify_args a = base_args(); a.tuning = &t;
        t.stats_split = 99; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG);
        t.stats_split = 0; t.stats_unroll = 3; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG);
        t.stats_unroll = 0; t.path = 9; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG);
        t.path = 0; t.fused_waves = 5; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG);
        t.fused_waves = 0; t.filter_path = 2; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG);
        t.filter_path = 0; t.tail_split = 3; EXPECT(hola_verify_ex(&a), HOLA_ERR_INVALID_ARG);
        t.tail_split = 0;
        for (int path = 0; path <= 3; ++path) {
            memset(&t, 0, sizeof t); t.path = path; t.stats_split = 4; t.stats_unroll = 4; t.fused_waves = 8;
            EXPECT_RAN(hola_verify_ex(&a));
        }
    }
    {   /* shapes that reach every launch sequence */
        hola_verify_args a = base_args();
        EXPECT_RAN(hola_verify_ex(&a));
        a.dtype = HOLA_DTYPE_F32; a.target_logits = (void*)0x1004; EXPECT_RAN(hola_verify_ex(&a));
        a = base_args(); a.B = 256; a.gamma = 8; a.V = 128256; EXPECT_RAN(hola_verify_ex(&a)); EXPECT_RAN(hola_verify_ex_static(&a));
        a.top_k = 50; a.top_p = 0.9f; EXPECT_RAN(hola_verify_ex(&a));
        EXPECT(hola_verify_ex_static(&a), HOLA_ERR_WORKSPACE);      /* the filtered headline batch outgrows the static array */
        a = base_args(); a.gamma = 63; a.V = 5; EXPECT_RAN(hola_verify_ex(&a));
        a = base_args(); a.draft_stats_in = (const double*)FAKE; a.target_stats_in = (const double*)FAKE; EXPECT_RAN(hola_verify_ex(&a));
        a = base_args(); a.temperature = 0.f; EXPECT_RAN(hola_verify_ex(&a));
        a = base_args(); a.V = 1 << 24; a.dtype = HOLA_DTYPE_F32; EXPECT_RAN(hola_verify_ex(&a));   /* more tiles than the tail kernel holds: path 3 */
        a = base_args(); EXPECT_RAN(hola_verify_literal_ex(&a, (int32_t*)FAKE, NULL));
        EXPECT(hola_verify_literal_ex(&a, NULL, NULL), HOLA_ERR_INVALID_ARG);
        EXPECT(hola_verify_literal_ex(NULL, (int32_t*)FAKE, NULL), HOLA_ERR_INVALID_ARG);
    }

    /* ---- short forms */
    EXPECT(hola_verify_bf16(NULL, FAKE, FAKE, 0, 2, 2, 10, 1.f, 1.f, FAKE, FAKE, FAKE, NULL), HOLA_ERR_INVALID_ARG);
    EXPECT(hola_verify_f32(FAKE, FAKE, FAKE, 0, 2, 0, 10, 1.f, 1.f, FAKE, FAKE, FAKE, NULL), HOLA_ERR_INVALID_ARG);
    EXPECT(hola_verify_f32(FAKE, FAKE, FAKE, 0, 2, 2, 10, 0.f, 1.f, FAKE, FAKE, FAKE, NULL), HOLA_ERR_INVALID_ARG);
    EXPECT(hola_verify_bf16(FAKE, FAKE, FAKE, 0, 0, 2, 10, 1.f, 1.f, FAKE, FAKE, FAKE, NULL), HOLA_OK);

    /* ---- hierarchy */
    {
        const float taus[2] = {1.f, 2.f};
        hola_model_logits m[3];
        memset(m, 0, sizeof m);
        EXPECT(hola_hsd_verify(m, 3, HOLA_DTYPE_BF16, FAKE, 0, 0, 4, 2, 10, NULL, 1.f, taus, FAKE, FAKE, FAKE, NULL, WS, (size_t)1 << 30, NULL),
               HOLA_ERR_INVALID_ARG);
        for (int i = 0; i < 3; ++i) m[i].logits = FAKE;
        EXPECT(hola_hsd_verify(m, 3, HOLA_DTYPE_BF16, FAKE, 0, 0, 4, 2, 10, NULL, 1.f, taus, FAKE, FAKE, FAKE, NULL, WS, 16, NULL), HOLA_ERR_WORKSPACE);
        EXPECT(hola_hsd_verify(m, 1, HOLA_DTYPE_BF16, FAKE, 0, 0, 4, 2, 10, NULL, 1.f, taus, FAKE, FAKE, FAKE, NULL, WS, (size_t)1 << 30, NULL),
               HOLA_ERR_INVALID_ARG);
        EXPECT_RAN(hola_hsd_verify(m, 3, HOLA_DTYPE_BF16, FAKE, 0, 0, 4, 2, 10, NULL, 1.f, taus, FAKE, FAKE, FAKE, NULL, WS, (size_t)1 << 30, NULL));
        EXPECT(hola_hsd_verify_ex(NULL), HOLA_ERR_INVALID_ARG);
    }

    /* ---- token trees */
    EXPECT(hola_verify_tree(NULL), HOLA_ERR_INVALID_ARG);
    { hola_tree_args a = base_tree(); a.N = 64; EXPECT(hola_verify_tree(&a), HOLA_ERR_INVALID_ARG); }
    { hola_tree_args a = base_tree(); a.node_parent = NULL; EXPECT(hola_verify_tree(&a), HOLA_ERR_INVALID_ARG); }
    { hola_tree_args a = base_tree(); a.temperature = 0.f; EXPECT(hola_verify_tree(&a), HOLA_ERR_UNSUPPORTED); }
    { hola_tree_args a = base_tree(); a.V = 1 << 23; a.dtype = HOLA_DTYPE_F32; EXPECT(hola_verify_tree(&a), HOLA_ERR_UNSUPPORTED); }
    { hola_tree_args a = base_tree(); a.workspace_bytes = 4096; EXPECT(hola_verify_tree(&a), HOLA_ERR_WORKSPACE); }
    { hola_tree_args a = base_tree(); a.B = 0; EXPECT(hola_verify_tree(&a), HOLA_OK); }
    { hola_tree_args a = base_tree(); EXPECT_RAN(hola_verify_tree(&a)); a.N = 63; a.B = 300; EXPECT_RAN(hola_verify_tree(&a)); }

    /* ---- statistics entries, aids */
    EXPECT(hola_row_stats(NULL, 0, 0, 4, 10, 1.f, (double*)FAKE, WS, (size_t)1 << 30, NULL), HOLA_ERR_INVALID_ARG);
    EXPECT(hola_row_stats(FAKE, 0, 0, 4, 10, 0.f, (double*)FAKE, WS, (size_t)1 << 30, NULL), HOLA_ERR_INVALID_ARG);
    EXPECT(hola_row_stats(FAKE, 0, 0, 0, 10, 1.f, (double*)FAKE, WS, (size_t)1 << 30, NULL), HOLA_OK);
    EXPECT_RAN(hola_row_stats(FAKE, 0, 0, 4, 10, 1.f, (double*)FAKE, WS, (size_t)1 << 30, NULL));
    EXPECT_RAN(hola_tile_stats(FAKE, HOLA_DTYPE_BF16, 0, 4, 100, 32, 1.f, (double*)FAKE, WS, (size_t)1 << 30, NULL));
    EXPECT(hola_tile_stats(FAKE, HOLA_DTYPE_BF16, 0, 4, 100, 0, 1.f, (double*)FAKE, WS, (size_t)1 << 30, NULL), HOLA_ERR_INVALID_ARG);
    EXPECT_RAN(hola_merge_tile_stats((const double*)FAKE, 4, 3, (double*)FAKE, NULL));
    EXPECT(hola_set_tuning(NULL), HOLA_OK);
    { hola_tuning t; memset(&t, 0, sizeof t); t.stats_unroll = 3; EXPECT(hola_set_tuning(&t), HOLA_ERR_INVALID_ARG);
      t.stats_unroll = 16; t.stats_split = 16; t.path = 3; EXPECT(hola_set_tuning(&t), HOLA_OK); EXPECT(hola_set_tuning(NULL), HOLA_OK); }
    {
        double ms[HOLA_N_STAGES]; int64_t n[HOLA_N_STAGES];
        int32_t stage[8]; float lms[8]; int64_t cnt = -1;
        memset(ms, 0, sizeof ms); memset(n, 0, sizeof n);
        EXPECT(hola_profile_enable(1), HOLA_OK);
        { hola_verify_args a = base_args(); EXPECT_RAN(hola_verify_ex(&a)); }
        EXPECT_RAN(hola_profile_collect(ms, n));
        EXPECT_RAN(hola_profile_collect_launches(stage, lms, 8, &cnt));
        CHECK(cnt >= 0);
        EXPECT(hola_profile_enable(0), HOLA_OK);
    }
    EXPECT_RAN(hola_copy_bytes(FAKE, FAKE, 4096, NULL));
    EXPECT_RAN(hola_read_probe(FAKE, 1 << 20, 1 << 17, 1, 1, NULL));
    hola_shutdown();
    printf("failures=%d rc=%d\n", failures, failures ? 1 : 0);
    return failures ? 1 : 0;
}
