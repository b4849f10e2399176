/* A caller of libopttree written in plain C against include/opttree.h and the HIP runtime only (no PyTorch, no
 * Python): reads one decoding step's inputs from a file, runs ot_build_tree and ot_tree_verify_attention with the
 * mask of the tree just built, writes the outputs to a file.  tests/test_zy_c_caller.py writes the inputs with
 * the seeded generators, runs this program and compares what it wrote with the oracle.  TEST INFRASTRUCTURE.
 *
 * usage: abi_client IN OUT
 * IN : int32 batch, vocab, depth, k, n, dtype, q_heads, kv_heads, head_dim, max_prefix;  int32 prefix_len[batch];
 *      logits [batch][depth][n][vocab]; Q [batch][q_heads][n][D]; K_prefix, V_prefix [batch][kv_heads][max_prefix][D];
 *      K_tree, V_tree [batch][kv_heads][n][D]  (elements of `dtype`: 0 = f32, 1 = bf16; all dense)
 * OUT: token, parent, depth int32 [batch][n]; score float [batch][n]; mask uint64 [batch][n][W]; n_out int32 [batch];
 *      expect double [batch]; O [batch][q_heads][n][D] in `dtype`
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "opttree.h"

#define CHECK_HIP(x)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (x);                                                                \
        if (e_ != hipSuccess) {                                                             \
            fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));      \
            return 2;                                                                       \
        }                                                                                   \
    } while (0)
#define CHECK_OT(x)                                                                         \
    do {                                                                                    \
        int s_ = (x);                                                                       \
        if (s_ != OT_OK) {                                                                  \
            fprintf(stderr, "%s:%d: %s (hip error %d)\n", __FILE__, __LINE__, ot_status_string(s_), \
                    ot_last_hip_error());                                                   \
            return 3;                                                                       \
        }                                                                                   \
    } while (0)

/* read `bytes` from the file into a fresh device buffer */
static int upload(FILE* f, size_t bytes, void** dev) {
    void* host = malloc(bytes ? bytes : 1);
    if (!host || fread(host, 1, bytes, f) != bytes) { fprintf(stderr, "short input file\n"); return 1; }
    if (hipMalloc(dev, bytes ? bytes : 16) != hipSuccess) return 1;
    if (hipMemcpy(*dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return 1;
    free(host);
    return 0;
}

static int download(FILE* f, const void* dev, size_t bytes) {
    void* host = malloc(bytes ? bytes : 1);
    if (!host) return 1;
    if (hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost) != hipSuccess) return 1;
    if (fwrite(host, 1, bytes, f) != bytes) return 1;
    free(host);
    return 0;
}

int main(int argc, char** argv) {
    if (argc != 3) { fprintf(stderr, "usage: %s IN OUT\n", argv[0]); return 1; }
    FILE* in = fopen(argv[1], "rb");
    if (!in) { perror(argv[1]); return 1; }
    int32_t h[10];
    if (fread(h, sizeof(int32_t), 10, in) != 10) { fprintf(stderr, "short header\n"); return 1; }
    const int batch = h[0], vocab = h[1], depth = h[2], k = h[3], n = h[4], dtype = h[5];
    const int q_heads = h[6], kv_heads = h[7], D = h[8], max_prefix = h[9];
    const size_t es = dtype == OT_BF16 ? 2 : 4;
    const size_t W = OT_MASK_WORDS(n);
    printf("libopttree %d: batch %d vocab %d depth %d k %d n %d; %d/%d heads of %d, prefix up to %d\n", ot_version(),
           batch, vocab, depth, k, n, q_heads, kv_heads, D, max_prefix);

    void *prefix_len, *logits, *Q, *Kp, *Vp, *Kt, *Vt;
    if (upload(in, (size_t)batch * 4, &prefix_len) || upload(in, (size_t)batch * depth * n * vocab * es, &logits) ||
        upload(in, (size_t)batch * q_heads * n * D * es, &Q) ||
        upload(in, (size_t)batch * kv_heads * max_prefix * D * es, &Kp) ||
        upload(in, (size_t)batch * kv_heads * max_prefix * D * es, &Vp) ||
        upload(in, (size_t)batch * kv_heads * n * D * es, &Kt) || upload(in, (size_t)batch * kv_heads * n * D * es, &Vt))
        return 2;
    fclose(in);

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));

    /* ---- the draft tree ---- */
    ot_build_params bp;
    memset(&bp, 0, sizeof(bp));
    bp.batch = batch; bp.vocab = vocab; bp.depth = depth; bp.k = k; bp.n = n; bp.logits_dtype = dtype;
    bp.stride_row = vocab; bp.stride_depth = (int64_t)n * vocab; bp.stride_seq = (int64_t)depth * n * vocab;
    const size_t bws_bytes = ot_build_workspace_bytes(&bp);
    if (!bws_bytes) { fprintf(stderr, "shape not supported by ot_build_tree\n"); return 3; }
    void* bws;
    CHECK_HIP(hipMalloc(&bws, bws_bytes));
    ot_tree_out out;
    CHECK_HIP(hipMalloc((void**)&out.token, (size_t)batch * n * 4));
    CHECK_HIP(hipMalloc((void**)&out.parent, (size_t)batch * n * 4));
    CHECK_HIP(hipMalloc((void**)&out.depth, (size_t)batch * n * 4));
    CHECK_HIP(hipMalloc((void**)&out.score, (size_t)batch * n * 4));
    CHECK_HIP(hipMalloc((void**)&out.mask, (size_t)batch * n * W * 8));
    CHECK_HIP(hipMalloc((void**)&out.n_out, (size_t)batch * 4));
    CHECK_HIP(hipMalloc((void**)&out.expect, (size_t)batch * 8));
    CHECK_OT(ot_build_tree(&bp, logits, bws, bws_bytes, &out, stream));

    /* ---- the target's attention over the tree, masked by the tree just built (same stream: ordered) ---- */
    ot_attn_params ap;
    memset(&ap, 0, sizeof(ap));
    ap.batch = batch; ap.q_heads = q_heads; ap.kv_heads = kv_heads; ap.head_dim = D; ap.n = n;
    ap.max_prefix = max_prefix; ap.dtype = dtype; ap.softmax_scale = 0.f; ap.n_keys = 0;
    const int64_t qs[3] = {(int64_t)q_heads * n * D, (int64_t)n * D, D};
    const int64_t ps[3] = {(int64_t)kv_heads * max_prefix * D, (int64_t)max_prefix * D, D};
    const int64_t ts[3] = {(int64_t)kv_heads * n * D, (int64_t)n * D, D};
    for (int i = 0; i < 3; ++i) {
        ap.q_strides[i] = ap.o_strides[i] = qs[i];
        ap.kp_strides[i] = ap.vp_strides[i] = ps[i];
        ap.kt_strides[i] = ap.vt_strides[i] = ts[i];
    }
    const size_t aws_bytes = ot_attn_workspace_bytes(&ap);
    if (!aws_bytes) { fprintf(stderr, "shape not supported by ot_tree_verify_attention\n"); return 3; }
    void *aws, *O;
    CHECK_HIP(hipMalloc(&aws, aws_bytes));
    CHECK_HIP(hipMalloc(&O, (size_t)batch * q_heads * n * D * es));
    CHECK_OT(ot_attn_workspace_prepare(aws, aws_bytes, stream));
    CHECK_OT(ot_tree_verify_attention(&ap, Q, Kp, Vp, Kt, Vt, (const int32_t*)prefix_len, out.mask, O, aws, aws_bytes,
                                      stream));
    CHECK_HIP(hipStreamSynchronize(stream));

    FILE* of = fopen(argv[2], "wb");
    if (!of) { perror(argv[2]); return 1; }
    if (download(of, out.token, (size_t)batch * n * 4) || download(of, out.parent, (size_t)batch * n * 4) ||
        download(of, out.depth, (size_t)batch * n * 4) || download(of, out.score, (size_t)batch * n * 4) ||
        download(of, out.mask, (size_t)batch * n * W * 8) || download(of, out.n_out, (size_t)batch * 4) ||
        download(of, out.expect, (size_t)batch * 8) || download(of, O, (size_t)batch * q_heads * n * D * es))
        return 2;
    fclose(of);
    printf("done\n");
    return 0;
}
