/* Host-side paths of libopttree under AddressSanitizer and UndefinedBehaviorSanitizer, on a machine without a GPU:
 * argument validation, workspace sizing and carving, the attention launch plan, the frontier-size tables.  Every call
 * here must come back with a status before anything is launched (invalid argument, unsupported shape, workspace too
 * small, scratch limit), or is a size query.  Built and run by tests/test_host_sanitizers.py against a host-only
 * build of the library's sources; prints "ok <calls>" when every status was the expected one. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "opttree.h"

static int calls = 0, bad = 0;
#define EXPECT(expr, want)                                                              \
    do {                                                                                \
        const long long got_ = (long long)(expr);                                       \
        ++calls;                                                                        \
        if (got_ != (long long)(want)) {                                                \
            ++bad;                                                                      \
            fprintf(stderr, "line %d: %s = %lld, expected %lld\n", __LINE__, #expr, got_, (long long)(want)); \
        }                                                                               \
    } while (0)

static ot_attn_params attn(int batch, int hq, int hkv, int d, int n, int maxp, int dtype, int nk) {
    ot_attn_params p;
    memset(&p, 0, sizeof p);
    p.batch = batch; p.q_heads = hq; p.kv_heads = hkv; p.head_dim = d; p.n = n; p.max_prefix = maxp; p.dtype = dtype;
    p.n_keys = nk;
    const int keys = nk > 0 ? nk : n;
    const int64_t q[3] = {(int64_t)hq * n * d, (int64_t)n * d, d};
    const int64_t kp[3] = {(int64_t)hkv * (maxp > 0 ? maxp : 1) * d, (int64_t)(maxp > 0 ? maxp : 1) * d, d};
    const int64_t kt[3] = {(int64_t)hkv * keys * d, (int64_t)keys * d, d};
    memcpy(p.q_strides, q, sizeof q); memcpy(p.o_strides, q, sizeof q);
    memcpy(p.kp_strides, kp, sizeof kp); memcpy(p.vp_strides, kp, sizeof kp);
    memcpy(p.kt_strides, kt, sizeof kt); memcpy(p.vt_strides, kt, sizeof kt);
    return p;
}

int main(void) {
    void* const f = (void*)0x1000;          /* a well-aligned pointer that is never dereferenced on the host */
    void* const odd = (void*)0x1002;

    /* ---- tree builder: sizes over a grid of shapes, then every rejection ---- */
    const int vocabs[] = {16, 100, 8192, 32000, 32768, 32769, 128256, 262144};
    const int ns[] = {1, 7, 50, 64, 65, 256};
    const int ks[] = {1, 8, 10, 16};
    const int depths[] = {1, 2, 10, 20, 32};
    for (unsigned a = 0; a < sizeof vocabs / sizeof *vocabs; ++a)
        for (unsigned b = 0; b < sizeof ns / sizeof *ns; ++b)
            for (unsigned c = 0; c < sizeof ks / sizeof *ks; ++c)
                for (unsigned d = 0; d < sizeof depths / sizeof *depths; ++d)
                    for (int dt = 0; dt < 2; ++dt) {
                        ot_build_params p = {3, vocabs[a], depths[d], ks[c], ns[b], dt, 0, 0, 0};
                        p.stride_row = vocabs[a]; p.stride_depth = (int64_t)ns[b] * vocabs[a];
                        p.stride_seq = p.stride_depth * depths[d];
                        const size_t need = ot_build_workspace_bytes(&p);
                        ++calls;
                        if (ks[c] > vocabs[a]) { if (need != 0) { ++bad; fprintf(stderr, "k > vocab accepted\n"); } continue; }
                        if (need == 0) { ++bad; fprintf(stderr, "valid build shape refused: V %d n %d k %d d %d\n", vocabs[a], ns[b], ks[c], depths[d]); continue; }
                        ot_tree_out out = {f, f, f, f, f, f, f};
                        EXPECT(ot_build_tree(&p, f, f, need - 1, &out, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                        EXPECT(ot_tree_begin(&p, f, need - 1, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                        EXPECT(ot_tree_expand(&p, 0, f, p.stride_seq, p.stride_row, f, need - 1, f, f, NULL, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                        EXPECT(ot_tree_finalize(&p, 1, f, need - 1, &out, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                        EXPECT(ot_tree_esub(&p, 1, 0.1, f, need - 1, f, f, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                        EXPECT(ot_tree_frontier_mask(&p, 1, f, need - 1, f, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                    }
    {
        ot_build_params p = {1, 1000, 4, 4, 16, 0, 64000, 16000, 1000};
        const size_t need = ot_build_workspace_bytes(&p);
        ot_tree_out out = {f, f, f, f, f, f, f};
        ot_build_params q;
        EXPECT(ot_build_workspace_bytes(NULL), 0);
        q = p; q.k = 17; EXPECT(ot_build_workspace_bytes(&q), 0);
        q = p; q.n = 257; EXPECT(ot_build_workspace_bytes(&q), 0);
        q = p; q.depth = 33; EXPECT(ot_build_workspace_bytes(&q), 0);
        q = p; q.batch = 0; EXPECT(ot_build_workspace_bytes(&q), 0);
        q = p; q.vocab = 262145; EXPECT(ot_build_workspace_bytes(&q), 0);
        q = p; q.logits_dtype = 7; EXPECT(ot_build_workspace_bytes(&q), 0);
        EXPECT(ot_build_tree(NULL, f, f, need, &out, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_build_tree(&p, NULL, f, need, &out, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_build_tree(&p, f, NULL, need, &out, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_build_tree(&p, f, f, need, NULL, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_build_tree(&p, f, odd, need, &out, NULL), OT_ERR_INVALID_ARG);
        q = p; q.stride_row = 999; EXPECT(ot_build_tree(&q, f, f, need, &out, NULL), OT_ERR_INVALID_ARG);
        ot_tree_out hole = out; hole.parent = NULL;
        EXPECT(ot_build_tree(&p, f, f, need, &hole, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_build_tree_timed(&p, f, f, need - 1, &out, NULL, NULL, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
        EXPECT(ot_build_tree_adaptive(&p, 0.1, f, f, need - 1, &out, f, f, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
        EXPECT(ot_build_tree_adaptive(&p, 0.1, f, f, need, &out, NULL, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_expand(&p, 4, f, 0, 1000, f, need, f, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_expand(&p, -1, f, 0, 1000, f, need, f, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_expand(&p, 0, f, 0, 999, f, need, f, f, NULL, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_expand(&p, 0, f, 0, 1000, f, need, f, NULL, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_expand(&p, 0, f, 0, 1000, f, need, f, f, odd, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_finalize(&p, 0, f, need, &out, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_finalize(&p, 5, f, need, &out, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_esub(&p, 0, 0.1, f, need, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_esub(&p, 1, 0.1, f, need, NULL, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_frontier_mask(&p, 0, f, need, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_frontier_mask(&p, 1, f, need, NULL, NULL), OT_ERR_INVALID_ARG);
    }

    /* ---- attention: the launch plan over a grid of shapes (sizes only), then the rejections ---- */
    const int heads[][2] = {{1, 1}, {4, 4}, {32, 32}, {40, 40}, {64, 8}, {32, 8}, {16, 2}, {8, 1}};
    const int prefixes[] = {0, 1, 63, 64, 1000, 4096, 8192, 100000};
    const int batches[] = {1, 3, 16, 32};
    const int nks[] = {0, 300, 768, 5120, 8192};
    for (unsigned a = 0; a < sizeof heads / sizeof *heads; ++a)
        for (unsigned b = 0; b < sizeof prefixes / sizeof *prefixes; ++b)
            for (unsigned c = 0; c < sizeof batches / sizeof *batches; ++c)
                for (unsigned d = 0; d < sizeof ns / sizeof *ns; ++d)
                    for (unsigned e = 0; e < sizeof nks / sizeof *nks; ++e)
                        for (int dt = 0; dt < 2; ++dt)
                            for (int hd = 64; hd <= 128; hd += 64) {
                                if (nks[e] && nks[e] < ns[d]) continue;
                                ot_attn_params p = attn(batches[c], heads[a][0], heads[a][1], hd, ns[d], prefixes[b], dt, nks[e]);
                                const size_t need = ot_attn_workspace_bytes(&p);
                                ++calls;
                                if (need < OT_ATTN_SYNC_BYTES) { ++bad; fprintf(stderr, "valid attention shape refused\n"); continue; }
                                void* kp = prefixes[b] ? f : NULL;
                                /* (for bf16 the size covers the 8-bit-cache variant's plan as well, which may be the larger
                                 * of the two: only the f32 size is tight for this call) */
                                EXPECT(ot_tree_verify_attention(&p, f, kp, kp, f, f, f, f, f, f, dt == 0 ? need - 1 : OT_ATTN_SYNC_BYTES, NULL),
                                       OT_ERR_WORKSPACE_TOO_SMALL);
                                if (dt == 1)
                                    EXPECT(ot_tree_verify_attention_fp8kv(&p, f, kp, kp, f, f, f, f, f, f, f, f, OT_ATTN_SYNC_BYTES, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                                if (need > OT_ATTN_SCRATCH_BYTES)
                                    EXPECT(ot_tree_verify_attention_noalloc(&p, f, kp, kp, f, f, f, f, f, NULL), OT_ERR_SCRATCH_LIMIT);
                            }
    {
        ot_attn_params p = attn(1, 4, 4, 64, 16, 128, 0, 0), q;
        const size_t need = ot_attn_workspace_bytes(&p);
        EXPECT(ot_attn_workspace_bytes(NULL), 0);
        q = p; q.q_heads = 6; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.head_dim = 96; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.n = 0; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.n = 257; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.n_keys = OT_MAX_TREE_KEYS + 1; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.n_keys = -1; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.max_prefix = -1; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.q_strides[2] = 62; EXPECT(ot_attn_workspace_bytes(&q), 0);
        q = p; q.kt_strides[0] = -64; EXPECT(ot_attn_workspace_bytes(&q), 0);
        EXPECT(ot_tree_verify_attention(NULL, f, f, f, f, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_verify_attention(&p, NULL, f, f, f, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_verify_attention(&p, f, NULL, f, f, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_verify_attention(&p, (void*)0x1008, f, f, f, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_verify_attention_timed(&p, f, f, f, f, f, f, f, f, f, need - 1, NULL, NULL, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
        EXPECT(ot_tree_verify_attention_fp8kv(&p, f, f, f, f, f, f, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);   /* f32 Q/O */
        q = attn(1, 4, 4, 64, 16, 128, 1, 0);
        EXPECT(ot_tree_verify_attention_fp8kv(&q, f, f, f, f, f, NULL, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_verify_attention_fp8kv(&q, f, f, f, f, f, f, odd, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        q.kp_strides[2] = 72;
        EXPECT(ot_tree_verify_attention_fp8kv(&q, f, f, f, f, f, f, f, f, f, f, f, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_tree_verify_attention_noalloc(NULL, f, f, f, f, f, f, f, f, NULL), OT_ERR_INVALID_ARG);
        q = p; q.head_dim = 96;
        EXPECT(ot_tree_verify_attention_noalloc(&q, f, f, f, f, f, f, f, f, NULL), OT_ERR_UNSUPPORTED);
        EXPECT(ot_attn_workspace_prepare(NULL, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_attn_workspace_prepare((void*)0x1008, need, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_attn_workspace_prepare(f, 100, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
        EXPECT(ot_kv_append(NULL, f, f, f, f, f, f, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_kv_append(&p, f, f, f, f, f, f, f, NULL, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_kv_append(&p, f, f, f, f, f, f, f, odd, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_kv_append(&p, f, f, f, f, f, f, f, f /* new_prefix_len == prefix_len */, NULL), OT_ERR_INVALID_ARG);
    }

    /* ---- verification ---- */
    for (unsigned a = 0; a < sizeof vocabs / sizeof *vocabs; ++a)
        for (unsigned b = 0; b < sizeof ns / sizeof *ns; ++b)
            for (int dt = 0; dt < 2; ++dt) {
                ot_verify_params p = {2, vocabs[a], ns[b], dt, (int64_t)(ns[b] + 1) * vocabs[a], vocabs[a]};
                const size_t need = ot_verify_workspace_bytes(&p);
                ++calls;
                if (need == 0) { ++bad; fprintf(stderr, "valid verify shape refused\n"); continue; }
                EXPECT(ot_verify_greedy(&p, f, f, f, f, f, need - 1, f, f, f, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
                const size_t need_s = ot_verify_sample_workspace_bytes(&p);
                ++calls;
                if (need_s) EXPECT(ot_verify_sample(&p, 1.0f, f, f, f, f, f, f, need_s - 1, f, f, f, NULL), OT_ERR_WORKSPACE_TOO_SMALL);
            }
    {
        ot_verify_params p = {1, 1000, 8, 0, 9000, 1000}, q;
        const size_t need = ot_verify_workspace_bytes(&p), need_s = ot_verify_sample_workspace_bytes(&p);
        EXPECT(ot_verify_workspace_bytes(NULL), 0);
        q = p; q.n = 0; EXPECT(ot_verify_workspace_bytes(&q), 0);
        q = p; q.stride_row = 999; EXPECT(ot_verify_workspace_bytes(&q), 0);
        EXPECT(ot_verify_greedy(&p, NULL, f, f, f, f, need, f, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_verify_greedy(&p, f, f, f, f, f, need, NULL, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_verify_sample(&p, 0.0f, f, f, f, f, f, f, need_s, f, f, f, NULL), OT_ERR_INVALID_ARG);
        EXPECT(ot_verify_sample(&p, 1.0f, f, NULL, f, f, f, f, need_s, f, f, f, NULL), OT_ERR_INVALID_ARG);
    }

    /* ---- the rest ---- */
    EXPECT(ot_yardstick_stream_read(NULL, 1 << 20, f, NULL), OT_ERR_INVALID_ARG);
    EXPECT(ot_yardstick_stream_read(f, 100, f, NULL), OT_ERR_INVALID_ARG);
    EXPECT(ot_yardstick_mfma_loop(0, f, NULL), OT_ERR_INVALID_ARG);
    EXPECT(ot_yardstick_stream_read_timed(f, 1 << 20, 0, f, NULL, NULL, NULL), OT_ERR_INVALID_ARG);
    for (int s = -7; s <= 1; ++s) { const char* m = ot_status_string(s); ++calls; if (!m || !*m) ++bad; }
    EXPECT(ot_version() > 0, 1);

    if (bad) { fprintf(stderr, "%d of %d checks failed\n", bad, calls); return 1; }
    printf("ok %d\n", calls);
    return 0;
}
