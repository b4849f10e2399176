// Tree selection: everything of Algorithm 1 that follows the row scan.
//   per drafting step t: candidate score = score(parent) + (x - lse)            (Eq. 2 in log space)
//                        keep the F_{t+1} = min(n, k F_t) best candidates       (Algorithm 1, "topk")
//                        number them by (parent slot, rank)
//   finally:             the n best nodes of the whole pool                     (Algorithm 1, last line)
//                        output order (depth, slot); parents, depths (= position offsets, Fig. 1),
//                        ancestor bitmask (Algorithm 2), E = sum of p^           (Eq. 3)
//
// One workgroup per sequence; lane j owns frontier slot j.  Scores are fp64 and compared
// through an order-preserving 64-bit integer key.  "Keep the best m of the workgroup's keys"
// never sorts: it finds the m-th largest key tau by pivoting (each round a lane proposes one
// of its keys still inside the open interval (lo, hi), the workgroup counts keys >= pivot and
// narrows the interval), then every lane keeps its keys > tau and ties at tau are handed out
// in index order.  Because each lane's candidates are already sorted by rank, the kept ones
// are a prefix per lane and the new slot numbering is an exclusive prefix sum of the counts.
#include "common.hpp"

namespace ot {
namespace {

typedef unsigned long long u64;

struct SelKArgs {
    const double* row_lse; const float* row_topv; const int32_t* row_topi;
    int k, n, depth, rows_per_seq;
    int F[OT_MAX_DEPTH + 2];
    int row_start[OT_MAX_DEPTH + 2];
    u64* pool_key; int32_t* pool_tok; int32_t* pool_par;      // [batch][depth][n]  (streaming state)
    ot_tree_out out;
    int32_t* frontier_token; int32_t* frontier_parent;        // [batch][n]         (streaming step)
    int step;
};

__device__ __forceinline__ int wave_sum_i(int v) {
    v += dpp_i<DPP_QUAD_XOR1>(v, v);
    v += dpp_i<DPP_QUAD_XOR2>(v, v);
    v += dpp_i<DPP_ROW_HALF_MIRROR>(v, v);
    v += dpp_i<DPP_ROW_MIRROR>(v, v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// Workgroup collectives.  SINGLE: the workgroup is one wavefront, no LDS and no barrier needed.
template <bool SINGLE>
struct Group {
    int* red;        // LDS int[2][4]
    u64* bc;         // LDS u64[2]
    int* scan;       // LDS int[2][4]
    int phase, bphase, sphase;
    int tid, wave, nw;

    __device__ int combine(int v, bool is_max) {
        if (SINGLE) return v;
        if ((tid & 63) == 0) red[phase * 4 + wave] = v;
        __syncthreads();
        int r = red[phase * 4];
        for (int w = 1; w < nw; ++w) r = is_max ? max(r, red[phase * 4 + w]) : r + red[phase * 4 + w];
        phase ^= 1;
        return r;
    }
    __device__ int max_i(int v) { return combine(wave_max_i(v), true); }
    __device__ int sum_i(int v) { return combine(wave_sum_i(v), false); }
    __device__ u64 bcast(u64 v, int src) {
        if (SINGLE) return __shfl(v, src);
        if (tid == src) bc[bphase] = v;
        __syncthreads();
        const u64 r = bc[bphase];
        bphase ^= 1;
        return r;
    }
    // exclusive prefix sum over the workgroup in thread order
    __device__ int excl_scan(int v) {
        const int lane = tid & 63;
        int inc = v;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(inc, o);
            if (lane >= o) inc += up;
        }
        if (SINGLE) return inc - v;
        if (lane == 63) scan[sphase * 4 + wave] = inc;
        __syncthreads();
        int off = 0;
        for (int w = 0; w < wave; ++w) off += scan[sphase * 4 + w];
        sphase ^= 1;
        return inc - v + off;
    }
};

// tau = the `want`-th largest of the workgroup's keys (M per lane; key 0 = absent).
// Returns per lane the number of its keys > tau and == tau, and the workgroup totals.
template <int M, bool SINGLE>
__device__ void select_threshold(const u64 (&key)[M], int want, Group<SINGLE>& g, u64& tau, int& lane_gt, int& lane_eq,
                                 int& total_gt, int& total_eq) {
    u64 lo = 0ull, hi = ~0ull;
    int a = 0, bgt = 0, bge = M;
#pragma unroll
    for (int r = 0; r < M; ++r) bgt += key[r] > 0ull ? 1 : 0;
    int f_hi = 0;
    int tot_gt_lo = g.sum_i(bgt);
    int tot_ge_lo = 0x7fffffff;
    // every round removes at least the pivot from the open interval, so M * blockDim rounds always
    // suffice; the bound makes termination unconditional
    for (int round = 0; round < M * 256 + 2; ++round) {
        const int in_range = tot_gt_lo - f_hi;
        if (in_range <= 0) break;
        const int cnt = bgt - a;
        const int target = want - f_hi;
        int q = 0;
        if (cnt > 0) {
            q = (int)(((long long)cnt * (2 * target - 1)) / (2 * in_range));
            q = q > cnt - 1 ? cnt - 1 : q;
        }
        u64 prop = 0ull;
        int ord = 0;
#pragma unroll
        for (int r = 0; r < M; ++r) {
            const bool inr = key[r] > lo && key[r] < hi;
            if (inr && ord == q) prop = key[r];
            ord += inr ? 1 : 0;
        }
        const int packed = cnt > 0 ? ((cnt << 16) | (0xffff - g.tid)) : 0;
        const int win = g.max_i(packed);
        const int src = 0xffff - (win & 0xffff);
        const u64 p = g.bcast(prop, src);
        int gge = 0, ggt = 0;
#pragma unroll
        for (int r = 0; r < M; ++r) {
            gge += key[r] >= p ? 1 : 0;
            ggt += key[r] > p ? 1 : 0;
        }
        const int both = g.sum_i(gge | (ggt << 16));
        const int f_p = both & 0xffff, gt_p = both >> 16;
        if (f_p >= want) { lo = p; bgt = ggt; bge = gge; tot_gt_lo = gt_p; tot_ge_lo = f_p; }
        else             { hi = p; a = gge; f_hi = f_p; }
    }
    tau = lo;
    lane_gt = a;
    lane_eq = bge - a;
    total_gt = f_hi;
    total_eq = tot_ge_lo - f_hi;
}

// One drafting step's cut: how many of this lane's (rank-sorted) candidates survive, and the
// first slot they occupy in the next layer.
template <int KMAX, bool SINGLE>
__device__ void layer_cut(const u64 (&ck)[KMAX], bool active, int k, int F, int want, Group<SINGLE>& g, int& cnt,
                          int& off) {
    if (k * F <= want) {
        cnt = active ? k : 0;
    } else {
        u64 tau; int lane_gt, lane_eq, total_gt, total_eq;
        select_threshold<KMAX, SINGLE>(ck, want, g, tau, lane_gt, lane_eq, total_gt, total_eq);
        const int need = want - total_gt;
        int take = lane_eq;
        if (total_eq != need) {           // ties at the cut: smaller parent slot first (ranks are contiguous per lane)
            const int before = g.excl_scan(lane_eq);
            take = need - before;
            take = take < 0 ? 0 : (take > lane_eq ? lane_eq : take);
        }
        cnt = lane_gt + take;
    }
    off = g.excl_scan(cnt);
}

struct RowData {
    double lse;
    float v[OT_MAX_TOPK];
    int i[OT_MAX_TOPK];
};

template <int KMAX>
__device__ __forceinline__ void load_row(const SelKArgs& a, long long rid, bool active, double& lse, float (&v)[KMAX],
                                         int (&id)[KMAX]) {
    lse = 0.0;
#pragma unroll
    for (int r = 0; r < KMAX; ++r) { v[r] = 0.f; id[r] = 0; }
    if (active) {
        lse = a.row_lse[rid];
#pragma unroll
        for (int r = 0; r < KMAX; ++r)
            if (r < a.k) { v[r] = a.row_topv[rid * a.k + r]; id[r] = a.row_topi[rid * a.k + r]; }
    }
}

// LDS carve-up shared by the kernels below.
struct Pool {
    u64* key;               // [D][NT]   key of pool node (layer t+1, slot)
    int* tok;               // [D][NT]
    unsigned short* par;    // [D][NT]   parent slot in the previous layer
    unsigned short* oidx;   // [D][NT]   output index of a selected node
    u64* mrow;              // [NT][4]   ancestor bitmask rows by output index
};
__device__ __forceinline__ Pool carve_pool(void* smem, int D, int NT) {
    Pool p;
    p.key = (u64*)smem;
    p.tok = (int*)(p.key + (size_t)D * NT);
    p.par = (unsigned short*)(p.tok + (size_t)D * NT);
    p.oidx = p.par + (size_t)D * NT;
    p.mrow = (u64*)(p.oidx + (size_t)D * NT);
    return p;
}
inline size_t pool_lds_bytes(int D, int NT) { return (size_t)D * NT * (8 + 4 + 2 + 2) + (size_t)NT * 4 * 8; }

// Last line of Algorithm 1 and the outputs.  `steps` layers are in the pool.
template <int DMAX, bool SINGLE>
__device__ void finalize_tree(const SelKArgs& a, const Pool& P, int steps, int b, Group<SINGLE>& g, int* s_cntw /*[OT_MAX_DEPTH][4]*/,
                              double* s_dsum /*[4]*/) {
    const int NT = blockDim.x, tid = threadIdx.x, n = a.n;
    const int W = OT_MASK_WORDS(n);
    int pool_nodes = 0;
    for (int t = 0; t < steps; ++t) pool_nodes += a.F[t + 1];
    const int n_out = pool_nodes < n ? pool_nodes : n;

    u64 pk[DMAX];
#pragma unroll
    for (int t = 0; t < DMAX; ++t) pk[t] = (t < steps && tid < a.F[t + 1]) ? P.key[t * NT + tid] : 0ull;

    unsigned int sel = 0;           // bit t: pool node (layer t+1, slot tid) is in the tree
    if (pool_nodes <= n) {
#pragma unroll
        for (int t = 0; t < DMAX; ++t) sel |= (pk[t] != 0ull ? 1u : 0u) << t;
    } else {
        u64 tau; int lane_gt, lane_eq, total_gt, total_eq;
        select_threshold<DMAX, SINGLE>(pk, n, g, tau, lane_gt, lane_eq, total_gt, total_eq);
#pragma unroll
        for (int t = 0; t < DMAX; ++t) sel |= (pk[t] > tau ? 1u : 0u) << t;
        int need = n - total_gt;
        if (total_eq == need) {
#pragma unroll
            for (int t = 0; t < DMAX; ++t) sel |= (pk[t] == tau ? 1u : 0u) << t;
        } else {                     // ties at the cut: shallower first, then smaller slot
            for (int t = 0; t < steps; ++t) {
                u64 kt = 0ull;
#pragma unroll
                for (int tt = 0; tt < DMAX; ++tt) kt = (tt == t) ? pk[tt] : kt;
                const int eq = kt == tau ? 1 : 0;
                const int before = g.excl_scan(eq);
                const int layer_eq = g.sum_i(eq);
                if (eq && before < need) sel |= 1u << t;
                need -= layer_eq < need ? layer_eq : need;
            }
        }
    }

    // output index = rank in (depth, slot) order among the selected nodes
    const int lane = tid & 63;
    int my_prefix[DMAX];
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {
        const u64 bal = __ballot((sel >> t) & 1u);
        my_prefix[t] = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0 && t < steps) s_cntw[t * 4 + g.wave] = __popcll(bal);
    }
    __syncthreads();
    {
        int base = 0;
#pragma unroll
        for (int t = 0; t < DMAX; ++t) {
            if (t < steps) {
                int mine = base;
                for (int w = 0; w < g.nw; ++w) {
                    const int c = s_cntw[t * 4 + w];
                    if (w < g.wave) mine += c;
                    base += c;
                }
                if ((sel >> t) & 1u) P.oidx[t * NT + tid] = (unsigned short)(mine + my_prefix[t]);
            }
        }
    }
    __syncthreads();

    // ancestor masks, layer by layer (a parent's row is complete before its children read it)
    for (int t = 0; t < steps; ++t) {
        if ((sel >> t) & 1u) {
            const int i = P.oidx[t * NT + tid];
            u64 row[4] = {0ull, 0ull, 0ull, 0ull};
            if (t > 0) {
                const int pi = P.oidx[(t - 1) * NT + P.par[t * NT + tid]];
#pragma unroll
                for (int w = 0; w < 4; ++w) row[w] = P.mrow[pi * 4 + w];
            }
            row[i >> 6] |= 1ull << (i & 63);
#pragma unroll
            for (int w = 0; w < 4; ++w) P.mrow[i * 4 + w] = row[w];
        }
        __syncthreads();
    }

    // emit
    const size_t ob = (size_t)b * n;
    double e_sum = 0.0;
    for (int t = 0; t < steps; ++t) {
        if ((sel >> t) & 1u) {
            const int i = P.oidx[t * NT + tid];
            const double sc = key_f64(P.key[t * NT + tid]);
            a.out.token[ob + i] = P.tok[t * NT + tid];
            a.out.parent[ob + i] = t == 0 ? -1 : (int)P.oidx[(t - 1) * NT + P.par[t * NT + tid]];
            a.out.depth[ob + i] = t + 1;
            a.out.score[ob + i] = (float)sc;
            for (int w = 0; w < W; ++w) a.out.mask[(ob + i) * W + w] = P.mrow[i * 4 + w];
            e_sum += exp(sc);
        }
    }
    for (int i = n_out + tid; i < n; i += NT) {
        a.out.token[ob + i] = -1;
        a.out.parent[ob + i] = -1;
        a.out.depth[ob + i] = 0;
        a.out.score[ob + i] = -INFINITY;
        for (int w = 0; w < W; ++w) a.out.mask[(ob + i) * W + w] = 0ull;
    }
    e_sum = wave_sum(e_sum);
    if (lane == 0) s_dsum[g.wave] = e_sum;
    __syncthreads();
    if (tid == 0) {
        double e = 0.0;
        for (int w = 0; w < g.nw; ++w) e += s_dsum[w];
        a.out.expect[b] = e;
        a.out.n_out[b] = n_out;
    }
}

#define OT_SELECT_SHARED                                   \
    extern __shared__ u64 smem[];                          \
    __shared__ int s_red[8];                               \
    __shared__ u64 s_bc[2];                                \
    __shared__ int s_scan[8];                              \
    __shared__ int s_cntw[OT_MAX_DEPTH * 4];               \
    __shared__ double s_dsum[4];                           \
    Group<SINGLE> g;                                       \
    g.red = s_red; g.bc = s_bc; g.scan = s_scan;           \
    g.phase = g.bphase = g.sphase = 0;                     \
    g.tid = threadIdx.x; g.wave = threadIdx.x >> 6; g.nw = blockDim.x >> 6;

// One-shot: all steps in one launch, pool resident in LDS.
template <int KMAX, int DMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_oneshot_kernel(const SelKArgs a) {
    OT_SELECT_SHARED
    const int NT = blockDim.x, tid = threadIdx.x, b = blockIdx.x, D = a.depth;
    const Pool P = carve_pool(smem, D, NT);

    double lse, nlse;
    float v[KMAX], nv[KMAX];
    int id[KMAX], nid[KMAX];
    load_row<KMAX>(a, (long long)b * a.rows_per_seq + tid, tid < a.F[0], nlse, nv, nid);
    for (int t = 0; t < D; ++t) {
        const int F = a.F[t], Fn = a.F[t + 1];
        const bool active = tid < F;
        lse = nlse;
#pragma unroll
        for (int r = 0; r < KMAX; ++r) { v[r] = nv[r]; id[r] = nid[r]; }
        if (t + 1 < D)   // next step's row: its address does not depend on the tree, fetch it now
            load_row<KMAX>(a, (long long)b * a.rows_per_seq + a.row_start[t + 1] + tid, tid < Fn, nlse, nv, nid);
        const double S = (t == 0 || !active) ? 0.0 : key_f64(P.key[(t - 1) * NT + tid]);
        u64 ck[KMAX];
#pragma unroll
        for (int r = 0; r < KMAX; ++r)
            ck[r] = (active && r < a.k) ? f64_key(S + ((double)v[r] - lse)) : 0ull;
        int cnt, off;
        layer_cut<KMAX, SINGLE>(ck, active, a.k, F, Fn, g, cnt, off);
#pragma unroll
        for (int r = 0; r < KMAX; ++r) {
            if (r < cnt) {
                P.key[t * NT + off + r] = ck[r];
                P.tok[t * NT + off + r] = id[r];
                P.par[t * NT + off + r] = (unsigned short)tid;
            }
        }
        __syncthreads();
    }
    finalize_tree<DMAX, SINGLE>(a, P, D, b, g, s_cntw, s_dsum);
}

// Streaming: one drafting step; the pool lives in the caller's workspace between launches.
template <int KMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_step_kernel(const SelKArgs a) {
    OT_SELECT_SHARED
    (void)smem; (void)s_cntw; (void)s_dsum;
    const int tid = threadIdx.x, b = blockIdx.x, t = a.step, n = a.n;
    const int F = a.F[t], Fn = a.F[t + 1];
    const bool active = tid < F;
    const size_t pb = (size_t)b * a.depth * n;
    double lse;
    float v[KMAX];
    int id[KMAX];
    load_row<KMAX>(a, (long long)b * a.rows_per_seq + tid, active, lse, v, id);
    const double S = (t == 0 || !active) ? 0.0 : key_f64(a.pool_key[pb + (size_t)(t - 1) * n + tid]);
    u64 ck[KMAX];
#pragma unroll
    for (int r = 0; r < KMAX; ++r) ck[r] = (active && r < a.k) ? f64_key(S + ((double)v[r] - lse)) : 0ull;
    int cnt, off;
    layer_cut<KMAX, SINGLE>(ck, active, a.k, F, Fn, g, cnt, off);
#pragma unroll
    for (int r = 0; r < KMAX; ++r) {
        if (r < cnt) {
            const size_t o = pb + (size_t)t * n + off + r;
            a.pool_key[o] = ck[r];
            a.pool_tok[o] = id[r];
            a.pool_par[o] = tid;
            a.frontier_token[(size_t)b * n + off + r] = id[r];
            a.frontier_parent[(size_t)b * n + off + r] = tid;
        }
    }
}

template <int DMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_finalize_kernel(const SelKArgs a) {
    OT_SELECT_SHARED
    const int NT = blockDim.x, tid = threadIdx.x, b = blockIdx.x, n = a.n, steps = a.step;
    const Pool P = carve_pool(smem, a.depth, NT);
    const size_t pb = (size_t)b * a.depth * n;
    for (int t = 0; t < steps; ++t) {
        if (tid < a.F[t + 1]) {
            const size_t o = pb + (size_t)t * n + tid;
            P.key[t * NT + tid] = a.pool_key[o];
            P.tok[t * NT + tid] = a.pool_tok[o];
            P.par[t * NT + tid] = (unsigned short)a.pool_par[o];
        }
    }
    __syncthreads();
    finalize_tree<DMAX, SINGLE>(a, P, steps, b, g, s_cntw, s_dsum);
}

SelKArgs make_args(const SelectGeometry& g, const BuildWorkspace& ws) {
    SelKArgs a;
    a.row_lse = ws.row_lse; a.row_topv = ws.row_topv; a.row_topi = ws.row_topi;
    a.k = g.k; a.n = g.n; a.depth = g.depth; a.rows_per_seq = g.rows_per_seq;
    for (int i = 0; i < OT_MAX_DEPTH + 2; ++i) { a.F[i] = g.F[i]; a.row_start[i] = g.row_start[i]; }
    a.pool_key = ws.pool_key; a.pool_tok = ws.pool_tok; a.pool_par = ws.pool_par;
    a.out = ot_tree_out{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    a.frontier_token = nullptr; a.frontier_parent = nullptr;
    a.step = 0;
    return a;
}

int threads_for(int n) { return ((n + 63) / 64) * 64; }

template <typename K>
int set_lds(K kernel, size_t bytes) {
    if (bytes > 64 * 1024) {
        if (bytes > 160 * 1024) return OT_ERR_UNSUPPORTED;
        OT_HIP_CHECK(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    }
    return OT_OK;
}

template <int KMAX, int DMAX, bool SINGLE>
int launch_oneshot_t(const SelKArgs& a, int batch, int NT, size_t lds, hipStream_t s) {
    int st = set_lds(tree_oneshot_kernel<KMAX, DMAX, SINGLE>, lds);
    if (st != OT_OK) return st;
    hipLaunchKernelGGL((tree_oneshot_kernel<KMAX, DMAX, SINGLE>), dim3(batch), dim3(NT), lds, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}
template <int KMAX, bool SINGLE>
int launch_oneshot_k(const SelKArgs& a, int batch, int NT, size_t lds, hipStream_t s) {
    if (a.depth <= 8) return launch_oneshot_t<KMAX, 8, SINGLE>(a, batch, NT, lds, s);
    if (a.depth <= 16) return launch_oneshot_t<KMAX, 16, SINGLE>(a, batch, NT, lds, s);
    return launch_oneshot_t<KMAX, 32, SINGLE>(a, batch, NT, lds, s);
}
template <bool SINGLE>
int launch_oneshot_s(const SelKArgs& a, int batch, int NT, size_t lds, hipStream_t s) {
    if (a.k <= 4) return launch_oneshot_k<4, SINGLE>(a, batch, NT, lds, s);
    if (a.k <= 8) return launch_oneshot_k<8, SINGLE>(a, batch, NT, lds, s);
    if (a.k <= 12) return launch_oneshot_k<12, SINGLE>(a, batch, NT, lds, s);
    return launch_oneshot_k<16, SINGLE>(a, batch, NT, lds, s);
}

template <int DMAX, bool SINGLE>
int launch_finalize_t(const SelKArgs& a, int batch, int NT, size_t lds, hipStream_t s) {
    int st = set_lds(tree_finalize_kernel<DMAX, SINGLE>, lds);
    if (st != OT_OK) return st;
    hipLaunchKernelGGL((tree_finalize_kernel<DMAX, SINGLE>), dim3(batch), dim3(NT), lds, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

}  // namespace

int launch_tree_oneshot(const SelectGeometry& g, const BuildWorkspace& ws, const ot_tree_out& out, hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.out = out;
    const int NT = threads_for(g.n);
    const size_t lds = pool_lds_bytes(g.depth, NT);
    return NT == 64 ? launch_oneshot_s<true>(a, g.batch, NT, lds, s) : launch_oneshot_s<false>(a, g.batch, NT, lds, s);
}

int launch_tree_step(const SelectGeometry& g, int step, const BuildWorkspace& ws, int32_t* frontier_token,
                     int32_t* frontier_parent, hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.step = step;
    a.frontier_token = frontier_token; a.frontier_parent = frontier_parent;
    const int NT = threads_for(g.n);
#define OT_STEP(KM)                                                                                         \
    do {                                                                                                    \
        if (NT == 64) hipLaunchKernelGGL((tree_step_kernel<KM, true>), dim3(g.batch), dim3(NT), 0, s, a);   \
        else          hipLaunchKernelGGL((tree_step_kernel<KM, false>), dim3(g.batch), dim3(NT), 0, s, a);  \
    } while (0)
    if (g.k <= 4) OT_STEP(4); else if (g.k <= 8) OT_STEP(8); else if (g.k <= 12) OT_STEP(12); else OT_STEP(16);
#undef OT_STEP
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

int launch_tree_finalize(const SelectGeometry& g, int steps_done, const BuildWorkspace& ws, const ot_tree_out& out,
                         hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.out = out;
    a.step = steps_done;
    const int NT = threads_for(g.n);
    const size_t lds = pool_lds_bytes(g.depth, NT);
    if (NT == 64) {
        if (steps_done <= 8) return launch_finalize_t<8, true>(a, g.batch, NT, lds, s);
        if (steps_done <= 16) return launch_finalize_t<16, true>(a, g.batch, NT, lds, s);
        return launch_finalize_t<32, true>(a, g.batch, NT, lds, s);
    }
    if (steps_done <= 8) return launch_finalize_t<8, false>(a, g.batch, NT, lds, s);
    if (steps_done <= 16) return launch_finalize_t<16, false>(a, g.batch, NT, lds, s);
    return launch_finalize_t<32, false>(a, g.batch, NT, lds, s);
}

}  // namespace ot
