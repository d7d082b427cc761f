// Host-side checks of libmoa under AddressSanitizer + UndefinedBehaviorSanitizer, on a machine without a GPU.
//
// Every entry point validates its arguments on the host before it launches anything, and moa_draft_step walks all
// of its stages once in a checks-only pass first (workspace carving, launch planning, pointer arithmetic on the
// caller's buffers).  This program drives exactly that code with device "pointers" that are never dereferenced: bad
// arguments must come back with their documented status, and well-formed calls must get through every host check and
// then fail at the first HIP call (no device) -- without the sanitizers seeing an out-of-bounds access, a misaligned
// access or an overflow on the way.  The gzip pass of the first message (Sec. 4.2) is host code throughout and is run
// for real.  Test infrastructure: built and run by a CPU test, never part of the library.
#include "../../include/moa.h"

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

static int failures = 0;

#define EXPECT(cond)                                                                      \
    do {                                                                                  \
        if (!(cond)) {                                                                    \
            printf("FAILED %s:%d: %s   (last error: %s)\n", __FILE__, __LINE__, #cond, moa_last_error()); \
            ++failures;                                                                   \
        }                                                                                 \
    } while (0)

// distinct, 256-byte aligned, never dereferenced
static void *fake(int n) { return (void *)(uintptr_t)(0x10000000ull + 0x100000ull * (unsigned)n); }

static moa_shape_t llama8b(int dtype) { return moa_shape_t{32, 4096, 32, 8, 128, 2048, 16, 8, dtype}; }

static void workspace_and_shapes()
{
    moa_shape_t s = llama8b(MOA_BF16);
    size_t n = 0, n2 = 0;
    EXPECT(moa_workspace_bytes(&s, 1, 1084, 60, 60, &n) == MOA_OK && n > 0);
    EXPECT(moa_workspace_bytes(&s, 16, 2048 + 64, 64, 1024, &n2) == MOA_OK && n2 > n);
    EXPECT(moa_workspace_bytes(&s, 8, 32768 + 128, 128, 8 * 128, &n2) == MOA_OK && n2 > n);
    EXPECT(moa_workspace_bytes(&s, 1, 1084, 60, 60, nullptr) == MOA_ERR_NULL);
    moa_shape_t bad = s;
    bad.n_kv_heads = 5;
    EXPECT(moa_workspace_bytes(&bad, 1, 1084, 60, 60, &n) == MOA_ERR_SHAPE);
    bad = s;
    bad.dtype = 9;
    EXPECT(moa_workspace_bytes(&bad, 1, 1084, 60, 60, &n) == MOA_ERR_DTYPE);
    EXPECT(moa_lsa_packed_weight_bytes(&s, &n) == MOA_OK && n == (size_t)(16 + 8 + 8) * 128 * 2048 * 2);
    moa_shape_t f32 = llama8b(MOA_F32);
    EXPECT(moa_lsa_packed_weight_bytes(&f32, &n) == MOA_ERR_SHAPE);
    moa_decoder_cfg_t cfg = {14336, 1e-5f, 5e5f};
    EXPECT(moa_tli_workspace_bytes(&s, &cfg, 1, 1084, 60, &n) == MOA_OK && n > 0);
    EXPECT(moa_mlp_block_workspace_bytes(MOA_BF16, 60, 4096, 7168, &n) == MOA_OK && n > 0);
    EXPECT(moa_linear_workspace_bytes(MOA_BF16, 60, 4096, 10240, &n) == MOA_OK);
}

static void single_entry_points()
{
    moa_shape_t s = llama8b(MOA_BF16);
    size_t ws = 0;
    moa_workspace_bytes(&s, 1, 1084, 60, 60, &ws);
    EXPECT(moa_tree_build(nullptr, 1, 8, nullptr, nullptr, nullptr, nullptr) == MOA_ERR_NULL);
    EXPECT(moa_tree_build((const int32_t *)fake(1), 1, MOA_MAX_TREE + 1, (uint64_t *)fake(2), (int32_t *)fake(3), nullptr, nullptr) == MOA_ERR_SHAPE);
    EXPECT(moa_lsa(&s, nullptr, 60, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), ws, nullptr) == MOA_ERR_NULL);
    EXPECT(moa_lsa(&s, fake(0), 60, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), 64, nullptr) == MOA_ERR_WORKSPACE);
    EXPECT(moa_lsa(&s, fake(0), -1, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), ws, nullptr) == MOA_ERR_SHAPE);
    EXPECT(moa_lsa(&s, fake(0), 0, fake(1), fake(2), fake(3), fake(4), fake(5), nullptr, 0, nullptr) == MOA_OK);
    EXPECT(moa_lsa_packed(&s, fake(0), 60, nullptr, fake(4), fake(5), fake(6), ws, nullptr) == MOA_ERR_NULL);
    EXPECT(moa_cross_attn_draft(&s, fake(0), 0, 60, fake(1), fake(2), fake(3), fake(4), (const int32_t *)fake(5), 1084, fake(6),
                                (int32_t *)fake(7), fake(8), ws, nullptr) == MOA_ERR_SHAPE);
    EXPECT(moa_tree_verify_attn(&s, fake(0), 1, 300, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), (const int32_t *)fake(7), 1084,
                                (const uint64_t *)fake(8), fake(9), fake(10), fake(11), (int32_t *)fake(12), fake(13), ws, nullptr) == MOA_ERR_SHAPE);
    // well-formed calls get through the host checks; without a device the first HIP call then fails
    int32_t rc = moa_lsa(&s, fake(0), 60, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), ws, nullptr);
    EXPECT(rc == MOA_ERR_HIP || rc == MOA_OK);
    rc = moa_tree_verify_attn(&s, fake(0), 1, 60, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), (const int32_t *)fake(7), 1084,
                              (const uint64_t *)fake(8), fake(9), fake(10), fake(11), (int32_t *)fake(12), fake(13), ws, nullptr);
    EXPECT(rc == MOA_ERR_HIP || rc == MOA_OK);
    rc = moa_tree_verify_attn_noalloc(&s, fake(0), 1, 60, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), (const int32_t *)fake(7),
                                      1084, (const uint64_t *)fake(8), fake(9), fake(10), fake(11), (int32_t *)fake(12), nullptr);
    EXPECT(rc == MOA_ERR_HIP || rc == MOA_OK);
    rc = moa_tree_verify_attn_noalloc(&s, fake(0), 8, 128, fake(1), fake(2), fake(3), fake(4), fake(5), fake(6), (const int32_t *)fake(7),
                                      32768 + 128, (const uint64_t *)fake(8), fake(9), fake(10), fake(11), (int32_t *)fake(12), nullptr);
    EXPECT(rc == MOA_ERR_WORKSPACE);            // more scratch than the fixed array holds
}

// a whole step with fake device pointers: the checks-only pass over every stage, under each schedule and regime
static void whole_step(int dtype, int B, int M, int P_cap, int64_t T_lsa, int layers, int schedule, bool with_sa, bool folded, bool packed,
                       bool tiny_ws)
{
    moa_shape_t s = llama8b(dtype), sa_shape = s;
    sa_shape.n_kv_heads = 4;
    size_t ws = 0;
    EXPECT(moa_workspace_bytes(&s, B, P_cap, M, T_lsa, &ws) == MOA_OK);
    std::vector<const void *> in[7];
    std::vector<void *> out[3];
    for (int l = 0; l < layers; ++l) {
        for (int k = 0; k < 7; ++k) in[k].push_back(fake(100 + 10 * l + k));
        for (int k = 0; k < 3; ++k) out[k].push_back(fake(100 + 10 * l + 7 + k));
    }
    moa_step_args_t a;
    memset(&a, 0, sizeof(a));
    a.shape = &s;
    a.B = B; a.M = M; a.Mq = M;
    a.parent = (const int32_t *)fake(1); a.mask = (uint64_t *)fake(2); a.depth = (int32_t *)fake(3);
    a.lsa_hs = fake(4); a.T_lsa = T_lsa;
    a.lsa_wq = fake(5); a.lsa_wk = fake(6); a.lsa_wv = fake(7); a.lsa_wo = fake(8); a.lsa_out = fake(9);
    a.tok_off = (const int32_t *)fake(10);
    a.ca_wk = fake(11); a.ca_wv = fake(12); a.ca_k = fake(13); a.ca_v = fake(14); a.ca_len = (int32_t *)fake(15); a.ca_P_cap = P_cap;
    a.ca_xq = fake(16); a.ca_wq = fake(17); a.ca_wo = fake(18); a.ca_out = fake(19);
    a.n_verify_layers = layers;
    a.v_x_host = in[0].data(); a.v_wq_host = in[1].data(); a.v_wk_host = in[2].data(); a.v_wv_host = in[3].data();
    a.v_wo_host = in[4].data(); a.v_kcache_host = in[5].data(); a.v_vcache_host = in[6].data();
    a.v_out_host = out[0].data(); a.v_ktree_host = out[1].data(); a.v_vtree_host = out[2].data();
    a.prefix_len = (const int32_t *)fake(20); a.P_cap = P_cap;
    a.tok = (const int32_t *)fake(21); a.tgt = (const int32_t *)fake(22);
    a.path = (int32_t *)fake(23); a.n_path = (int32_t *)fake(24); a.bonus = (int32_t *)fake(25);
    a.dev_status = (int32_t *)fake(26);
    a.ws = fake(60); a.ws_bytes = tiny_ws ? 1024 : ws;
    a.schedule = schedule;
    if (with_sa) {
        a.sa_shape = &sa_shape;
        a.sa_emb = fake(30); a.sa_wq = fake(31); a.sa_wk = fake(32); a.sa_wv = fake(33); a.sa_wo = fake(34);
        a.sa_kcache = fake(35); a.sa_vcache = fake(36); a.sa_P_cap = P_cap;
        a.sa_k_draft = fake(37); a.sa_v_draft = fake(38); a.sa_out = fake(39);
    }
    if (folded) { a.ca_wk_lsa_wo = fake(40); a.ca_wv_lsa_wo = fake(41); }
    if (packed) a.lsa_w_packed = fake(42);
    const int32_t rc = moa_draft_step(&a);
    if (tiny_ws) EXPECT(rc == MOA_ERR_WORKSPACE);
    else EXPECT(rc == MOA_ERR_HIP || rc == MOA_OK);
    moa_step_args_t b = a;                      // a NULL per-layer array is caught before any stage
    b.v_wo_host = nullptr;
    EXPECT(moa_draft_step(&b) == MOA_ERR_NULL);
    b = a;
    b.schedule = 7;
    EXPECT(moa_draft_step(&b) == MOA_ERR_SHAPE);
}

static void gzip_pass()
{
    std::vector<unsigned char> msg(50000);
    uint32_t x = 12345;
    for (size_t i = 0; i < msg.size(); ++i) { x = x * 1664525u + 1013904223u; msg[i] = (unsigned char)((x >> 24) % 37); }
    size_t bound = 0, n = 0, m = 0;
    EXPECT(moa_msg_gzip_bound(msg.size(), &bound) == MOA_OK && bound >= 18);
    std::vector<unsigned char> gz(bound), back(msg.size());
    EXPECT(moa_msg_gzip(msg.data(), msg.size(), gz.data(), gz.size(), &n) == MOA_OK && n > 18 && n < msg.size());
    EXPECT(moa_msg_gunzip(gz.data(), n, back.data(), back.size(), &m) == MOA_OK && m == msg.size());
    EXPECT(memcmp(msg.data(), back.data(), msg.size()) == 0);
    EXPECT(moa_msg_gunzip(gz.data(), n, back.data(), back.size() - 1, &m) == MOA_ERR_RANGE);
    EXPECT(moa_msg_gunzip(gz.data(), n - 9, back.data(), back.size(), &m) == MOA_ERR_SHAPE);
    EXPECT(moa_msg_gzip(msg.data(), msg.size(), gz.data(), 20, &n) == MOA_ERR_RANGE);
    EXPECT(moa_msg_gzip(nullptr, 0, gz.data(), gz.size(), &n) == MOA_OK);        // the empty message
    EXPECT(moa_msg_gunzip(gz.data(), n, nullptr, 0, &m) == MOA_OK && m == 0);
}

int main()
{
    workspace_and_shapes();
    single_entry_points();
    for (int schedule = MOA_SCHED_GROUPED; schedule <= MOA_SCHED_SEQUENTIAL; ++schedule) {
        whole_step(MOA_BF16, 1, 60, 1084, 60, 1, schedule, false, true, true, false);       // the headline step
        whole_step(MOA_BF16, 1, 60, 1084, 60, 3, schedule, true, false, false, false);      // Self-Attention layer in front, more layers
        whole_step(MOA_BF16, 1, 60, 1084, 1024, 1, schedule, false, true, true, false);     // first cycle: the whole prompt
        whole_step(MOA_BF16, 1, 60, 1084, 5, 1, schedule, false, true, true, false);        // accepted tokens only
        whole_step(MOA_BF16, 16, 64, 2048 + 64, 16 * 64, 1, schedule, false, true, true, false);
        whole_step(MOA_BF16, 8, 128, 32768 + 128, 8 * 128, 1, schedule, false, false, true, false);
        whole_step(MOA_F32, 2, 37, 300, 74, 2, schedule, false, false, false, false);
        whole_step(MOA_BF16, 1, 60, 1084, 60, 1, schedule, false, true, true, true);    // a workspace that is too small
    }
    gzip_pass();
    if (failures) {
        printf("host_check_driver: %d check(s) failed\n", failures);
        return 1;
    }
    printf("host_check_driver: ok\n");
    return 0;
}
