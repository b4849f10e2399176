// Greedy verification of a draft tree (Preliminaries, "Speculative Decoding"; Algorithm 2, "Verify"):
//   ground truth after a position = the target model's most probable token there;
//   the longest root branch of the tree that agrees with the ground truth is accepted, and the target's token
//   after the last accepted node is produced as well (A tokens for A - 1 accepted nodes);
//   the accepted nodes' K/V rows are appended to the cache.
// Three kernels: the row scan of the tree builder with k = 1 (arg-max of every target row; ties -> smaller
// token id), a walk down the tree (one workgroup per sequence, thread i = node i, one step per accepted
// node), and a row gather for the K/V append.
//
// Random sampling (Sec. 4, non-greedy settings): the paper changes only which tokens are acceptable and gives no
// rule; here the ground truth after a position is DRAWN from softmax(target logits / temperature) by the inverse
// CDF in token order of a caller-supplied uniform number, the walk is the same.  Two kernels replace the arg-max:
// sample_seg_kernel reads every row once and leaves (max, sum of exp) per segment of 64 lanes x 16 bytes;
// sample_pick_kernel (one wavefront per row) finds the segment in which the cumulative sum passes u x total and
// re-reads that one segment to find the token.
#include <string.h>

#include "common.hpp"

namespace ot {
namespace {

struct WalkKArgs {
    const int32_t* row_top;      // [batch][n + 1]  arg-max of the target's rows (row 0 = the root position)
    const int32_t *token, *parent, *n_out;
    int32_t *accept_len, *accept_node, *accept_token;
    int n;
};

// Thread i owns node i.  Children of one node carry distinct tokens, so at most one thread matches per step;
// the chain of matches is at most n_out long, which bounds the loop.
__global__ __launch_bounds__(256) void verify_walk_kernel(const WalkKArgs a) {
    __shared__ int s_next[2];
    const int b = blockIdx.x, i = threadIdx.x, n = a.n;
    const int n_out = a.n_out[b] < n ? a.n_out[b] : n;
    const bool have = i < n_out;
    const int my_tok = have ? a.token[(size_t)b * n + i] : -1;
    const int my_par = have ? a.parent[(size_t)b * n + i] : -2;
    const int32_t* top = a.row_top + (size_t)b * (n + 1);
    int cur = -1, A = 0;
    for (int step = 0; step <= n_out; ++step) {
        if (i == 0) s_next[step & 1] = -1;
        __syncthreads();
        const int g = top[cur + 1];                          // ground truth after `cur`
        if (have && my_par == cur && my_tok == g) s_next[step & 1] = i;
        __syncthreads();
        const int nx = s_next[step & 1];
        if (i == 0) {
            a.accept_token[(size_t)b * (n + 1) + A] = g;
            if (nx >= 0) a.accept_node[(size_t)b * n + A] = nx;
        }
        ++A;
        if (nx < 0) break;
        cur = nx;
    }
    // A tokens produced, A - 1 nodes accepted; the rest of the output rows is padding
    for (int j = A - 1 + i; j < n; j += blockDim.x) a.accept_node[(size_t)b * n + j] = -1;
    for (int j = A + i; j < n + 1; j += blockDim.x) a.accept_token[(size_t)b * (n + 1) + j] = -1;
    if (i == 0) a.accept_len[b] = A;
}

// ---------------------------------------------------------------------------------------------------------
// Drawing the ground truth at a temperature
// ---------------------------------------------------------------------------------------------------------
struct SampleKArgs {
    const void* logits;
    const float* u;              // [batch][n + 1]
    float* seg_m;                // [rows][nseg]   largest logit of the segment's wavefront (-inf: nothing finite)
    double* seg_s;               // [rows][nseg]   sum of exp2((x - seg_m) c) over the segment
    int32_t* truth;              // [rows]
    int rows_per_seq, vocab, nseg;
    long long stride_seq, stride_row;
    float c;                     // log2(e) / temperature
};

constexpr int kSegPerWave = 4;   // segments whose loads one wavefront keeps in flight

template <typename DT> struct SegOf { static constexpr int VEC = 16 / (int)sizeof(DT), ELEMS = 64 * VEC; };

// the VEC logits of one lane as floats; out-of-range elements read as -inf (probability 0)
template <typename DT, bool VECLOAD>
__device__ __forceinline__ void load_lane_elems(const DT* row, long long base, int vocab, float* v) {
    constexpr int VEC = SegOf<DT>::VEC;
    if (VECLOAD && base + VEC <= vocab) {
        const u32x4 w = *(const u32x4*)(row + base);
        if constexpr (sizeof(DT) == 2) {
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[2 * i] = bf16_lo(w[i]); v[2 * i + 1] = bf16_hi(w[i]); }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(w[i]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            float x = -INFINITY;
            if (base + i < vocab) {
                if constexpr (sizeof(DT) == 2) x = __uint_as_float((uint32_t)((const uint16_t*)row)[base + i] << 16);
                else x = ((const float*)row)[base + i];
            }
            v[i] = x;
        }
    }
}

__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// inclusive prefix sum over the lanes of a wavefront
__device__ __forceinline__ double wave_scan_f64(double v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}

// grid (segment groups, rows); every wavefront works alone: no LDS, no barrier
template <typename DT, bool VECLOAD>
__global__ __launch_bounds__(256) void sample_seg_kernel(const SampleKArgs a) {
    constexpr int VEC = SegOf<DT>::VEC, ELEMS = SegOf<DT>::ELEMS;
    const int row = blockIdx.y, b = row / a.rows_per_seq, j = row - b * a.rows_per_seq;
    const DT* x = (const DT*)a.logits + (long long)b * a.stride_seq + (long long)j * a.stride_row;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int seg0 = (blockIdx.x * 4 + wave) * kSegPerWave;
    if (seg0 >= a.nseg) return;
    float v[kSegPerWave][VEC];
#pragma unroll
    for (int s = 0; s < kSegPerWave; ++s)
        load_lane_elems<DT, VECLOAD>(x, (long long)(seg0 + s) * ELEMS + lane * VEC, a.vocab, v[s]);
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < kSegPerWave; ++s)
#pragma unroll
        for (int i = 0; i < VEC; ++i) m = fmaxf(m, v[s][i]);
    m = wave_max_f(m);
    const float mu = m == -INFINITY ? 0.f : m;
#pragma unroll
    for (int s = 0; s < kSegPerWave; ++s) {
        float e = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) e += __builtin_amdgcn_exp2f((v[s][i] - mu) * a.c);
        const double tot = wave_sum_f64((double)e);
        if (lane == 0 && seg0 + s < a.nseg) {
            a.seg_m[(size_t)row * a.nseg + seg0 + s] = m;
            a.seg_s[(size_t)row * a.nseg + seg0 + s] = tot;
        }
    }
}

// one wavefront per row; lane L owns the segments [L per, (L + 1) per)
template <typename DT, bool VECLOAD>
__global__ __launch_bounds__(64) void sample_pick_kernel(const SampleKArgs a) {
    constexpr int VEC = SegOf<DT>::VEC, ELEMS = SegOf<DT>::ELEMS;
    constexpr int PER_MAX = 8;
    const int row = blockIdx.x, b = row / a.rows_per_seq, j = row - b * a.rows_per_seq;
    const DT* x = (const DT*)a.logits + (long long)b * a.stride_seq + (long long)j * a.stride_row;
    const int lane = threadIdx.x;
    const int per = (a.nseg + 63) / 64;                    // <= PER_MAX, checked by the host
    const float* sm = a.seg_m + (size_t)row * a.nseg;
    const double* ss = a.seg_s + (size_t)row * a.nseg;
    float ms[PER_MAX];
    double w[PER_MAX];
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < PER_MAX; ++i) {
        const int s = lane * per + i;
        const bool ok = i < per && s < a.nseg;
        ms[i] = ok ? sm[s] : -INFINITY;
        w[i] = ok ? ss[s] : 0.0;
        M = fmaxf(M, ms[i]);
    }
    M = wave_max_f(M);
    if (M == -INFINITY) {                                  // no finite logit in the row: nothing to draw from
        if (lane == 0) a.truth[row] = 0;
        return;
    }
    double lane_sum = 0.0;
    double sc[PER_MAX];
#pragma unroll
    for (int i = 0; i < PER_MAX; ++i) {
        // weight of the segment relative to the row maximum (double exp2: relative error 1e-16)
        sc[i] = ms[i] == -INFINITY ? 0.0 : exp2(((double)ms[i] - (double)M) * (double)a.c);
        w[i] *= sc[i];
        lane_sum += w[i];
    }
    const double incl = wave_scan_f64(lane_sum, lane);
    const double total = __shfl(incl, 63);
    const double target = (double)a.u[row] * total;
    // first lane whose segments reach past the target; by rounding there may be none: the last lane with weight
    const unsigned long long past = __ballot(incl > target), any = __ballot(lane_sum > 0.0);
    const int L = past ? __ffsll((long long)past) - 1 : 63 - __clzll((long long)any);
    // inside lane L: the first segment that passes the target, else (rounding) the end of its last one with weight
    bool found = false;
    int seg = 0;
    float mseg = 0.f;
    double before = incl - lane_sum, rs = 0.0;                  // rs: residual in the segment's own units
#pragma unroll
    for (int i = 0; i < PER_MAX; ++i) {
        if (w[i] > 0.0 && !found) {
            seg = lane * per + i;
            mseg = ms[i];
            if (before + w[i] > target) { found = true; rs = (target - before) / sc[i]; }
            else rs = w[i] / sc[i];
        }
        if (!found) before += w[i];
    }
    seg = __shfl(seg, L);
    mseg = __shfl(mseg, L);
    rs = __shfl(rs, L);

    float v[VEC];
    load_lane_elems<DT, VECLOAD>(x, (long long)seg * ELEMS + lane * VEC, a.vocab, v);
    float e[VEC];
    double lane_e = 0.0;
#pragma unroll
    for (int i = 0; i < VEC; ++i) { e[i] = __builtin_amdgcn_exp2f((v[i] - mseg) * a.c); lane_e += (double)e[i]; }
    const double incl_e = wave_scan_f64(lane_e, lane);
    const unsigned long long past_e = __ballot(incl_e > rs), any_e = __ballot(lane_e > 0.0);
    const int Le = past_e ? __ffsll((long long)past_e) - 1 : 63 - __clzll((long long)any_e);
    if (lane == Le) {
        double acc = incl_e - lane_e;
        int k = -1, lastk = 0;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            acc += (double)e[i];
            if (e[i] > 0.f) { lastk = i; if (k < 0 && acc > rs) k = i; }
        }
        if (k < 0) k = lastk;
        a.truth[row] = seg * ELEMS + lane * VEC + k;
    }
}

template <typename DT, bool VECLOAD>
int launch_sample_t(const SampleKArgs& a, int rows, hipStream_t s) {
    const int groups = (a.nseg + 4 * kSegPerWave - 1) / (4 * kSegPerWave);
    hipLaunchKernelGGL((sample_seg_kernel<DT, VECLOAD>), dim3(groups, rows), dim3(256), 0, s, a);
    OT_HIP_CHECK(hipGetLastError());
    hipLaunchKernelGGL((sample_pick_kernel<DT, VECLOAD>), dim3(rows), dim3(64), 0, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

struct SampleWorkspace {
    float* seg_m;
    double* seg_s;
    int32_t* truth;
    size_t bytes;
    int nseg;
};

struct AppendKArgs {
    void *Kp, *Vp;
    const void *Kt, *Vt;
    const int32_t *prefix_len, *accept_len, *accept_node;
    int32_t* new_prefix_len;
    int kv_heads, n, D, max_prefix, esize;
    long long kps[3], vps[3], kts[3], vts[3];
};

// grid (accepted row j, batch x KV head); one wavefront copies the K row and the V row of node accept_node[j]
// to prefix row L + j, 16 bytes per lane
__global__ __launch_bounds__(64) void kv_append_kernel(const AppendKArgs a) {
    const int j = blockIdx.x, bh = blockIdx.y;
    const int b = bh / a.kv_heads, h = bh - b * a.kv_heads;
    int L = a.prefix_len[b];
    L = L < 0 ? 0 : (L > a.max_prefix ? a.max_prefix : L);
    const int cnt = a.accept_len[b] - 1;                     // accepted nodes
    if (j == 0 && h == 0 && threadIdx.x == 0) a.new_prefix_len[b] = L + cnt < a.max_prefix ? L + cnt : a.max_prefix;
    if (j >= cnt || L + j >= a.max_prefix) return;
    const int node = a.accept_node[(size_t)b * a.n + j];
    if (node < 0 || node >= a.n) return;
    const int chunks = a.D * a.esize / 16;                    // 16-byte chunks per row
    const int lane = threadIdx.x;
    const char* ks = (const char*)a.Kt + ((long long)b * a.kts[0] + (long long)h * a.kts[1] + (long long)node * a.kts[2]) * a.esize;
    const char* vs = (const char*)a.Vt + ((long long)b * a.vts[0] + (long long)h * a.vts[1] + (long long)node * a.vts[2]) * a.esize;
    char* kd = (char*)a.Kp + ((long long)b * a.kps[0] + (long long)h * a.kps[1] + (long long)(L + j) * a.kps[2]) * a.esize;
    char* vd = (char*)a.Vp + ((long long)b * a.vps[0] + (long long)h * a.vps[1] + (long long)(L + j) * a.vps[2]) * a.esize;
    for (int c = lane; c < chunks; c += 64) {
        *(u32x4*)(kd + 16 * c) = *(const u32x4*)(ks + 16 * c);
        *(u32x4*)(vd + 16 * c) = *(const u32x4*)(vs + 16 * c);
    }
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// row statistics of the (n + 1) target rows per sequence, k = 1
BuildWorkspace carve_verify_workspace(const ot_verify_params& p, void* base) {
    const size_t rows = (size_t)p.batch * (size_t)(p.n + 1);
    const size_t parts = (size_t)scan_parts(p.vocab);
    BuildWorkspace w;
    memset(&w, 0, sizeof(w));
    size_t off = 0;
    char* b = (char*)base;
    // (a null base is the sizing pass: offsets only)
    auto take = [&](size_t bytes) { char* q = b ? b + off : nullptr; off = align256(off + bytes); return (void*)q; };
    w.row_lse = (double*)take(rows * 8);
    w.row_topv = (float*)take(rows * 4);
    w.row_topi = (int32_t*)take(rows * 4);
    if (parts > 1) {
        w.part_m = (float*)take(rows * parts * 4);
        w.part_s = (double*)take(rows * parts * 8);
        w.part_topv = (float*)take(rows * parts * 4);
        w.part_topi = (int32_t*)take(rows * parts * 4);
    }
    w.bytes = off;
    return w;
}

SampleWorkspace carve_sample_workspace(const ot_verify_params& p, void* base) {
    const size_t rows = (size_t)p.batch * (size_t)(p.n + 1);
    const int elems = p.logits_dtype == OT_BF16 ? SegOf<uint16_t>::ELEMS : SegOf<float>::ELEMS;
    SampleWorkspace w;
    w.nseg = (p.vocab + elems - 1) / elems;
    size_t off = 0;
    char* b = (char*)base;
    // (a null base is the sizing pass: offsets only)
    auto take = [&](size_t bytes) { char* q = b ? b + off : nullptr; off = align256(off + bytes); return (void*)q; };
    w.seg_s = (double*)take(rows * w.nseg * 8);
    w.seg_m = (float*)take(rows * w.nseg * 4);
    w.truth = (int32_t*)take(rows * 4);
    w.bytes = off;
    return w;
}

int launch_walk(const ot_verify_params& p, const int32_t* row_top, const int32_t* token, const int32_t* parent,
                const int32_t* n_out, int32_t* accept_len, int32_t* accept_node, int32_t* accept_token, hipStream_t s) {
    WalkKArgs a;
    a.row_top = row_top; a.token = token; a.parent = parent; a.n_out = n_out;
    a.accept_len = accept_len; a.accept_node = accept_node; a.accept_token = accept_token; a.n = p.n;
    const int threads = (p.n + 63) / 64 * 64;
    hipLaunchKernelGGL(verify_walk_kernel, dim3(p.batch), dim3(threads), 0, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

int validate_verify(const ot_verify_params* p) {
    if (!p) return OT_ERR_INVALID_ARG;
    if (p->batch < 1 || p->vocab < 1 || p->n < 1) return OT_ERR_INVALID_ARG;
    if (p->logits_dtype != OT_F32 && p->logits_dtype != OT_BF16) return OT_ERR_INVALID_ARG;
    if (p->stride_row < p->vocab || p->stride_seq < 0) return OT_ERR_INVALID_ARG;
    if (p->n > OT_MAX_NODES || scan_parts(p->vocab) > 8) return OT_ERR_UNSUPPORTED;
    return OT_OK;
}

}  // namespace
}  // namespace ot

using namespace ot;

extern "C" {

size_t ot_verify_workspace_bytes(const ot_verify_params* p) {
    if (validate_verify(p) != OT_OK) return 0;
    return carve_verify_workspace(*p, nullptr).bytes;
}

int ot_verify_greedy(const ot_verify_params* p, const void* target_logits, const int32_t* token, const int32_t* parent,
                     const int32_t* n_out, void* workspace, size_t workspace_bytes, int32_t* accept_len,
                     int32_t* accept_node, int32_t* accept_token, void* hip_stream) {
    int st = validate_verify(p);
    if (st != OT_OK) return st;
    if (!target_logits || !token || !parent || !n_out || !workspace || !accept_len || !accept_node || !accept_token)
        return OT_ERR_INVALID_ARG;
    if ((uintptr_t)workspace % 16) return OT_ERR_INVALID_ARG;
    const int esize = p->logits_dtype == OT_BF16 ? 2 : 4;
    if ((uintptr_t)target_logits % esize) return OT_ERR_INVALID_ARG;
    const void* ip[6] = {token, parent, n_out, accept_len, accept_node, accept_token};
    for (int i = 0; i < 6; ++i)
        if ((uintptr_t)ip[i] % 4) return OT_ERR_INVALID_ARG;
    const BuildWorkspace ws = carve_verify_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)hip_stream;

    ScanGeometry sg;
    sg.batch = p->batch; sg.vocab = p->vocab; sg.k = 1; sg.dtype = p->logits_dtype;
    sg.nsteps = 1; sg.rows_per_seq = p->n + 1;
    sg.grow_k = 1; sg.grow_n = 1;
    sg.stride_seq = p->stride_seq; sg.stride_depth = 0; sg.stride_row = p->stride_row;
    st = launch_row_scan(sg, target_logits, ws, s);
    if (st != OT_OK) return st;

    return launch_walk(*p, ws.row_topi, token, parent, n_out, accept_len, accept_node, accept_token, s);
}

size_t ot_verify_sample_workspace_bytes(const ot_verify_params* p) {
    if (validate_verify(p) != OT_OK) return 0;
    const SampleWorkspace w = carve_sample_workspace(*p, nullptr);
    return w.nseg > 64 * 8 ? 0 : w.bytes;
}

int ot_verify_sample(const ot_verify_params* p, float temperature, const void* target_logits, const float* u,
                     const int32_t* token, const int32_t* parent, const int32_t* n_out, void* workspace,
                     size_t workspace_bytes, int32_t* accept_len, int32_t* accept_node, int32_t* accept_token,
                     void* hip_stream) {
    int st = validate_verify(p);
    if (st != OT_OK) return st;
    if (!(temperature > 0.f) || !(temperature <= 3.0e38f)) return OT_ERR_INVALID_ARG;
    if (!target_logits || !u || !token || !parent || !n_out || !workspace || !accept_len || !accept_node || !accept_token)
        return OT_ERR_INVALID_ARG;
    if ((uintptr_t)workspace % 16) return OT_ERR_INVALID_ARG;
    const int esize = p->logits_dtype == OT_BF16 ? 2 : 4;
    if ((uintptr_t)target_logits % esize) return OT_ERR_INVALID_ARG;
    const void* ip[7] = {u, token, parent, n_out, accept_len, accept_node, accept_token};
    for (int i = 0; i < 7; ++i)
        if ((uintptr_t)ip[i] % 4) return OT_ERR_INVALID_ARG;
    const SampleWorkspace ws = carve_sample_workspace(*p, workspace);
    if (ws.nseg > 64 * 8) return OT_ERR_UNSUPPORTED;          // segments per lane of the picking wavefront
    if ((long long)p->batch * (p->n + 1) > 65535) return OT_ERR_UNSUPPORTED;
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)hip_stream;

    SampleKArgs a;
    a.logits = target_logits; a.u = u; a.seg_m = ws.seg_m; a.seg_s = ws.seg_s; a.truth = ws.truth;
    a.rows_per_seq = p->n + 1; a.vocab = p->vocab; a.nseg = ws.nseg;
    a.stride_seq = p->stride_seq; a.stride_row = p->stride_row;
    a.c = (float)(1.4426950408889634 / (double)temperature);
    const int rows = p->batch * (p->n + 1);
    // 16-byte loads need every row to start on a 16-byte boundary
    const int vec = 16 / esize;
    const bool vecload = (uintptr_t)target_logits % 16 == 0 && p->stride_seq % vec == 0 && p->stride_row % vec == 0;
    if (p->logits_dtype == OT_BF16)
        st = vecload ? launch_sample_t<uint16_t, true>(a, rows, s) : launch_sample_t<uint16_t, false>(a, rows, s);
    else
        st = vecload ? launch_sample_t<float, true>(a, rows, s) : launch_sample_t<float, false>(a, rows, s);
    if (st != OT_OK) return st;
    return launch_walk(*p, ws.truth, token, parent, n_out, accept_len, accept_node, accept_token, s);
}

int ot_kv_append(const ot_attn_params* p, void* K_prefix, void* V_prefix, const void* K_tree, const void* V_tree,
                 const int32_t* prefix_len, const int32_t* accept_len, const int32_t* accept_node,
                 int32_t* new_prefix_len, void* hip_stream) {
    if (!p) return OT_ERR_INVALID_ARG;
    if (p->batch < 1 || p->kv_heads < 1 || p->n < 1 || p->max_prefix < 1 || p->head_dim < 1) return OT_ERR_INVALID_ARG;
    if (p->dtype != OT_F32 && p->dtype != OT_BF16) return OT_ERR_INVALID_ARG;
    if (p->n > OT_MAX_NODES) return OT_ERR_UNSUPPORTED;
    if ((long long)p->batch * p->kv_heads > 65535) return OT_ERR_UNSUPPORTED;
    const int esize = p->dtype == OT_BF16 ? 2 : 4;
    if ((p->head_dim * esize) % 16) return OT_ERR_UNSUPPORTED;
    if (!K_prefix || !V_prefix || !K_tree || !V_tree || !prefix_len || !accept_len || !accept_node || !new_prefix_len)
        return OT_ERR_INVALID_ARG;
    const void* vp[4] = {K_prefix, V_prefix, K_tree, V_tree};
    for (int i = 0; i < 4; ++i)
        if ((uintptr_t)vp[i] % 16) return OT_ERR_INVALID_ARG;
    if (((uintptr_t)prefix_len % 4) || ((uintptr_t)accept_len % 4) || ((uintptr_t)accept_node % 4) ||
        ((uintptr_t)new_prefix_len % 4))
        return OT_ERR_INVALID_ARG;
    {   // the copying workgroups read prefix_len[b] while new_prefix_len[b] is written: the arrays must be disjoint
        const uintptr_t a0 = (uintptr_t)prefix_len, b0 = (uintptr_t)new_prefix_len, len = (uintptr_t)p->batch * 4;
        if (a0 < b0 + len && b0 < a0 + len) return OT_ERR_INVALID_ARG;
    }
    const int vec = 16 / esize;
    const int64_t* strides[4] = {p->kp_strides, p->vp_strides, p->kt_strides, p->vt_strides};
    for (int t = 0; t < 4; ++t) {
        for (int i = 0; i < 3; ++i)
            if (strides[t][i] < 0 || strides[t][i] % vec) return OT_ERR_INVALID_ARG;
        if (strides[t][2] < p->head_dim) return OT_ERR_INVALID_ARG;
    }
    AppendKArgs a;
    a.Kp = K_prefix; a.Vp = V_prefix; a.Kt = K_tree; a.Vt = V_tree;
    a.prefix_len = prefix_len; a.accept_len = accept_len; a.accept_node = accept_node; a.new_prefix_len = new_prefix_len;
    a.kv_heads = p->kv_heads; a.n = p->n; a.D = p->head_dim; a.max_prefix = p->max_prefix; a.esize = esize;
    for (int i = 0; i < 3; ++i) {
        a.kps[i] = p->kp_strides[i]; a.vps[i] = p->vp_strides[i]; a.kts[i] = p->kt_strides[i]; a.vts[i] = p->vt_strides[i];
    }
    // at most n nodes can be accepted; rows beyond a sequence's accepted count end at once
    hipLaunchKernelGGL(kv_append_kernel, dim3(p->n, p->batch * p->kv_heads), dim3(64), 0, (hipStream_t)hip_stream, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

}  // extern "C"
