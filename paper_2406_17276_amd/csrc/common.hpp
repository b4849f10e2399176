// Internal declarations shared by the translation units of libopttree (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "opttree.h"

namespace ot {

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
void set_last_hip_error(int e);

#define OT_HIP_CHECK(expr)                                   \
    do {                                                     \
        hipError_t e__ = (expr);                             \
        if (e__ != hipSuccess) {                             \
            ::ot::set_last_hip_error((int)e__);              \
            return OT_ERR_HIP;                               \
        }                                                    \
    } while (0)

// Frontier sizes F_0 = 1, F_{t+1} = min(n, k F_t) and their prefix sums
// (Algorithm 1: each drafting step keeps at most n candidates).
struct Frontier {
    int F[OT_MAX_DEPTH + 2];          // F[t], t = 0..depth
    int row_start[OT_MAX_DEPTH + 2];  // rows scanned before step t
    int rows;                         // rows per sequence over `depth` steps
    int pool;                         // nodes per sequence = sum_{t=1..depth} F[t]
};
Frontier make_frontier(int k, int n, int depth);

// Elements of one vocabulary row handled by one workgroup of the row scan.
constexpr int kScanPartElems = 32768;
inline int scan_parts(int vocab) { return (vocab + kScanPartElems - 1) / kScanPartElems; }

// Workspace of the tree builder (device memory, caller-owned), carved by the host.
struct BuildWorkspace {
    double* row_lse;                // [rows_total]
    float* row_topv;                // [rows_total][k]
    int32_t* row_topi;              // [rows_total][k]
    float* part_m;                  // [rows_total][P]        (P > 1 only)
    double* part_s;                 // [rows_total][P]
    float* part_topv;               // [rows_total][P][k]
    int32_t* part_topi;             // [rows_total][P][k]
    double* pool_key;               // [batch][depth][n]   streaming state: log p^ of every pool node
    double* step_tau;               // [batch][depth]      streaming state: cut value of every step
    int32_t* pool_tok;              // [batch][depth][n]
    int32_t* pool_par;              // [batch][depth][n]
    double* pool_p;                 // [batch][depth][n]   streaming state: p^ of every pool node
    double* seq_E;                  // [batch]             streaming state: E of Algorithm 1's loop
    int32_t* seq_steps;             // [batch]             layers drafted (frozen when the loop has stopped)
    int32_t* seq_active;            // [batch]             0 once E_sub - E <= delta was seen
    unsigned short* front_anc;      // [2][batch][n][OT_MAX_DEPTH]  root paths (pool indices) of the last two frontiers
    size_t bytes;
};
BuildWorkspace carve_build_workspace(const ot_build_params& p, void* base);

// Which logits rows a scan launch covers: a sequence's rows are those of `nsteps` steps, step t holding F_t rows
// with F_0 = 1 and F_{t+1} = min(grow_n, grow_k F_t) (the frontier sizes of Algorithm 1; nsteps = 1 with
// rows_per_seq rows: one plain block of rows).  Row (b, t, j) is at base + b*ss + t*sd + j*sr.
struct ScanGeometry {
    int batch, vocab, k, dtype;
    int nsteps;                       // steps covered by this launch
    int rows_per_seq;
    int grow_k, grow_n;               // frontier growth; unused when nsteps == 1
    long long stride_seq, stride_depth, stride_row;
};

// ev0/ev1 (optional): events that receive the begin and end time stamps of the scan kernel itself
// skip_frozen: rows of sequences whose ws.seq_active flag is 0 (stopped by the rule of Algorithm 1) are not read
int launch_row_scan(const ScanGeometry& g, const void* logits, const BuildWorkspace& ws, hipStream_t s,
                    hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr, bool skip_frozen = false);

struct SelectGeometry {
    int batch, k, n, depth;
    int rows_per_seq;
    int F[OT_MAX_DEPTH + 2];
    int row_start[OT_MAX_DEPTH + 2];
};
int launch_tree_oneshot(const SelectGeometry& g, const BuildWorkspace& ws, const ot_tree_out& out, hipStream_t s);
int launch_tree_step(const SelectGeometry& g, int step, const BuildWorkspace& ws, int32_t* frontier_token,
                     int32_t* frontier_parent, int32_t* frontier_count, hipStream_t s);
int launch_tree_finalize(const SelectGeometry& g, int steps_done, const BuildWorkspace& ws, const ot_tree_out& out,
                         hipStream_t s);
int launch_tree_begin(const SelectGeometry& g, const BuildWorkspace& ws, hipStream_t s);
bool tree_adaptive_supported(const SelectGeometry& g);
int launch_tree_adaptive(const SelectGeometry& g, double delta, const BuildWorkspace& ws, const ot_tree_out& out,
                         int32_t* steps_used, double* e_sub, hipStream_t s);
int launch_tree_front_mask(const SelectGeometry& g, int steps_done, const BuildWorkspace& ws, uint64_t* mask_out,
                           int mask_words, hipStream_t s);
int launch_tree_esub(const SelectGeometry& g, int steps_done, double delta, const BuildWorkspace& ws, double* e_sub,
                     int32_t* go_on, hipStream_t s);

struct AttnPlan {
    int row_blocks;      // blocks of query rows per KV head
    int splits;          // KV splits per (b, kv head, row block)
    int balance;         // bf16 batches: workgroups take their jobs longest first, decided on the device
    size_t part_o_bytes, part_ml_bytes, bytes;
};
AttnPlan plan_attention(const ot_attn_params& p, bool kv8 = false);
int launch_tree_attention(const ot_attn_params& p, const AttnPlan& plan, const void* Q, const void* Kp, const void* Vp,
                          const void* Kt, const void* Vt, const int32_t* prefix_len, const uint64_t* mask, void* O,
                          void* workspace, hipStream_t s, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr,
                          const float* k_scale = nullptr, const float* v_scale = nullptr);

}  // namespace ot

// ---------------------------------------------------------------------------
// device side helpers
// ---------------------------------------------------------------------------
#if defined(__HIPCC__)
namespace ot {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Order-preserving map from double to uint64: a > b  <=>  key(a) > key(b) (no NaNs).
__device__ __forceinline__ unsigned long long f64_key(double v) {
    unsigned long long u = (unsigned long long)__double_as_longlong(v);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double key_f64(unsigned long long k) {
    unsigned long long u = (k >> 63) ? (k & 0x7fffffffffffffffull) : ~k;
    return __longlong_as_double((long long)u);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// DPP moves inside a 64-lane wavefront (GCN/CDNA encodings).
// BOUND (bound_ctrl): a lane whose source does not exist reads 0 instead of keeping `old`.  The quad and mirror
// permutations have a source for every lane, so the flag changes nothing there -- except that the compiler may
// then fold the move into the instruction that uses it.
template <int CTRL, int ROW_MASK = 0xf, bool BOUND = (ROW_MASK == 0xf && (CTRL < 0x100 || CTRL == 0x140 || CTRL == 0x141))>
__device__ __forceinline__ int dpp_i(int old, int v) {
    return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, BOUND);
}
constexpr int DPP_QUAD_XOR1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_MIRROR = 0x140;
constexpr int DPP_ROW_BCAST15 = 0x142;
constexpr int DPP_ROW_BCAST31 = 0x143;

// max over each row of 16 lanes, result in every lane of the row
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, __int_as_float(dpp_i<DPP_QUAD_XOR1>(__float_as_int(v), __float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_i<DPP_QUAD_XOR2>(__float_as_int(v), __float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_i<DPP_ROW_HALF_MIRROR>(__float_as_int(v), __float_as_int(v))));
    v = fmaxf(v, __int_as_float(dpp_i<DPP_ROW_MIRROR>(__float_as_int(v), __float_as_int(v))));
    return v;
}
// max over the 64 lanes of the wavefront, result in every lane
__device__ __forceinline__ float wave_max(float v) {
    v = row16_max(v);
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ int wave_max_i(int v) {
    v = max(v, dpp_i<DPP_QUAD_XOR1>(v, v));
    v = max(v, dpp_i<DPP_QUAD_XOR2>(v, v));
    v = max(v, dpp_i<DPP_ROW_HALF_MIRROR>(v, v));
    v = max(v, dpp_i<DPP_ROW_MIRROR>(v, v));
    v = max(v, __shfl_xor(v, 16));
    v = max(v, __shfl_xor(v, 32));
    return v;
}

// ---- wavefront reductions that end in a scalar (DPP inside rows of 16, v_readlane across rows) ----
__device__ __forceinline__ int rl(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float rl_f(float v, int lane) { return __int_as_float(rl(__float_as_int(v), lane)); }
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
    const int lo = dpp_i<CTRL>(0, __double2loint(v));
    const int hi = dpp_i<CTRL>(0, __double2hiint(v));
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double rl_d(double v, int lane) {
    return __hiloint2double(rl(__double2hiint(v), lane), rl(__double2loint(v), lane));
}
__device__ __forceinline__ double wave_sum_d(double v) {
    v += dpp_d<DPP_QUAD_XOR1>(v);
    v += dpp_d<DPP_QUAD_XOR2>(v);
    v += dpp_d<DPP_ROW_HALF_MIRROR>(v);
    v += dpp_d<DPP_ROW_MIRROR>(v);
    return (rl_d(v, 0) + rl_d(v, 16)) + (rl_d(v, 32) + rl_d(v, 48));
}
// sum over the wavefront as a scalar: fp32 inside each row of 16 lanes, the four row sums added in fp64
__device__ __forceinline__ double wave_sum_rows_d(float v) {
    v += __int_as_float(dpp_i<DPP_QUAD_XOR1>(__float_as_int(v), __float_as_int(v)));
    v += __int_as_float(dpp_i<DPP_QUAD_XOR2>(__float_as_int(v), __float_as_int(v)));
    v += __int_as_float(dpp_i<DPP_ROW_HALF_MIRROR>(__float_as_int(v), __float_as_int(v)));
    v += __int_as_float(dpp_i<DPP_ROW_MIRROR>(__float_as_int(v), __float_as_int(v)));
    return ((double)rl_f(v, 0) + (double)rl_f(v, 16)) + ((double)rl_f(v, 32) + (double)rl_f(v, 48));
}
// max over the wavefront as a scalar
__device__ __forceinline__ float wave_max_f(float v) {
    v = row16_max(v);
    return fmaxf(fmaxf(rl_f(v, 0), rl_f(v, 16)), fmaxf(rl_f(v, 32), rl_f(v, 48)));
}

}  // namespace ot
#endif
