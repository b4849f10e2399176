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
    int r0[OT_MAX_DEPTH + 2];      // rank whose per-lane minimum is a lower bound of step t's cut
    double* pool_key; int32_t* pool_tok; int32_t* pool_par;   // [batch][depth][n]  (streaming state)
    double* step_tau;                                         // [batch][depth]     (streaming state)
    double* pool_p;                                           // [batch][depth][n]  (streaming state) p^ of every pool node
    double* seq_E; int32_t* seq_steps; int32_t* seq_active;   // [batch]            (streaming state) adaptive depth
    double* e_sub; int32_t* go_on; double delta;              // outputs / threshold of the E_sub query
    unsigned short* front_anc;                                // [2][batch][n][OT_MAX_DEPTH] (streaming state): the pool
                                                              // indices of every node of the last two frontiers' root
                                                              // paths, the node itself last
    u64* mask_out; int mask_words;                            // output of the frontier-mask query
    int gridDim_batch;                                        // batch size (the grid of these kernels)
    int32_t* steps_used;                                      // [batch] output of the one-shot adaptive build
    ot_tree_out out;
    int32_t* frontier_token; int32_t* frontier_parent;        // [batch][n]         (streaming step)
    int32_t* frontier_count;                                  // [batch] or null    (streaming step)
    int step;
    int rehearse;                                             // fast kernel: 1 if the launch has LDS for the rehearsing wavefront
};

__device__ __forceinline__ double nan_d() { return __longlong_as_double(0x7ff8000000000000ll); }   // "absent"

// ---- integer wavefront reductions that end in a scalar ----
__device__ __forceinline__ int wave_max_u(int v) {
    v = max(v, dpp_i<DPP_QUAD_XOR1>(v, v));
    v = max(v, dpp_i<DPP_QUAD_XOR2>(v, v));
    v = max(v, dpp_i<DPP_ROW_HALF_MIRROR>(v, v));
    v = max(v, dpp_i<DPP_ROW_MIRROR>(v, v));
    return max(max(rl(v, 0), rl(v, 16)), max(rl(v, 32), rl(v, 48)));
}
__device__ __forceinline__ int wave_sum_u(int v) {
    v += dpp_i<DPP_QUAD_XOR1>(v, v);
    v += dpp_i<DPP_QUAD_XOR2>(v, v);
    v += dpp_i<DPP_ROW_HALF_MIRROR>(v, v);
    v += dpp_i<DPP_ROW_MIRROR>(v, v);
    return (rl(v, 0) + rl(v, 16)) + (rl(v, 32) + rl(v, 48));
}
// fmin/fmax ignore NaN operands, NaN marks "absent"
__device__ __forceinline__ double wave_min_d(double v) {
    v = fmin(v, dpp_d<DPP_QUAD_XOR1>(v));
    v = fmin(v, dpp_d<DPP_QUAD_XOR2>(v));
    v = fmin(v, dpp_d<DPP_ROW_HALF_MIRROR>(v));
    v = fmin(v, dpp_d<DPP_ROW_MIRROR>(v));
    return fmin(fmin(rl_d(v, 0), rl_d(v, 16)), fmin(rl_d(v, 32), rl_d(v, 48)));
}
// inclusive prefix sum inside the wavefront: Kogge-Stone inside rows (row_shr, zero fill), then row totals
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    const int t0 = rl(v, 15), t1 = rl(v, 31), t2 = rl(v, 47);
    const int row = lane >> 4;
    return v + (row > 0 ? t0 : 0) + (row > 1 ? t1 : 0) + (row > 2 ? t2 : 0);
}

// Barrier that orders LDS traffic only.  __syncthreads() would also wait for the global loads that
// prefetch the next step's row statistics; nothing here communicates through global memory.
template <bool SINGLE>
__device__ __forceinline__ void lds_sync() {
    if (SINGLE) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    else        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Workgroup collectives.  SINGLE: the workgroup is one wavefront, no LDS and no barrier needed.
template <bool SINGLE>
struct Group {
    int* red;        // LDS int[2][4]
    double* bc;      // LDS double[2]
    double* redd;    // LDS double[2][4]
    int phase, bphase, dphase;
    int tid, lane, wave, nw;
    int nt;          // threads of the group = stride of its LDS key tables

    __device__ __forceinline__ int combine(int v, bool is_max) {
        if (SINGLE) return v;
        if (lane == 0) red[phase * 4 + wave] = v;
        lds_sync<false>();
        int r = red[phase * 4];
        for (int w = 1; w < nw; ++w) r = is_max ? max(r, red[phase * 4 + w]) : r + red[phase * 4 + w];
        phase ^= 1;
        return r;
    }
    __device__ __forceinline__ int max_i(int v) { return combine(wave_max_u(v), true); }
    __device__ __forceinline__ int sum_i(int v) { return combine(wave_sum_u(v), false); }
    __device__ __forceinline__ double min_d(double v) {
        v = wave_min_d(v);
        if (SINGLE) return v;
        if (lane == 0) redd[dphase * 4 + wave] = v;
        lds_sync<false>();
        double r = redd[dphase * 4];
        for (int w = 1; w < nw; ++w) r = fmin(r, redd[dphase * 4 + w]);
        dphase ^= 1;
        return r;
    }
    __device__ __forceinline__ double sum_d(double v) {
        v = wave_sum_d(v);
        if (SINGLE) return v;
        if (lane == 0) redd[dphase * 4 + wave] = v;
        lds_sync<false>();
        double r = redd[dphase * 4];
        for (int w = 1; w < nw; ++w) r += redd[dphase * 4 + w];
        dphase ^= 1;
        return r;
    }
    // value of thread `src` (uniform) for everybody
    __device__ __forceinline__ double bcast(double v, int src) {
        if (SINGLE) return rl_d(v, src);
        if (tid == src) bc[bphase] = v;
        lds_sync<false>();
        const double r = bc[bphase];
        bphase ^= 1;
        return r;
    }
    // exclusive prefix sum over the workgroup in thread order
    __device__ __forceinline__ int excl_scan(int v) {
        const int inc = wave_incl_scan(v, lane);
        if (SINGLE) return inc - v;
        if (lane == 63) red[phase * 4 + wave] = inc;
        lds_sync<false>();
        int off = 0;
        for (int w = 0; w < wave; ++w) off += red[phase * 4 + w];
        phase ^= 1;
        return inc - v + off;
    }
};

constexpr int kBuckets = 256;

// next double above v (v finite)
__device__ __forceinline__ double next_up(double v) {
    if (v == 0.0) return __longlong_as_double(1ll);
    const long long bits = __double_as_longlong(v);
    return __longlong_as_double(v > 0.0 ? bits + 1 : bits - 1);
}

// Sort M doubles in registers, descending, NaN last (Batcher's odd-even merge network).
template <int M>
__device__ __forceinline__ void sort_desc(double (&x)[M]) {
#pragma unroll
    for (int p = 1; p < M; p *= 2)
#pragma unroll
        for (int k = p; k >= 1; k /= 2)
#pragma unroll
            for (int j = k % p; j <= M - 1 - k; j += 2 * k)
#pragma unroll
                for (int i = 0; i < k; ++i)
                    if (i + j + k <= M - 1 && (i + j) / (2 * p) == (i + j + k) / (2 * p)) {
                        const double u = x[i + j], w = x[i + j + k];
                        const bool swap = !(u >= w) && (w == w);
                        x[i + j] = swap ? w : u;
                        x[i + j + k] = swap ? u : w;
                    }
}

// Exact end game of a selection, on keys sorted per lane (descending, NaN last): ks[a..b) are this lane's
// keys still inside the range, f_hi keys of the workgroup lie above the range, f_lo lie above or inside it,
// every key inside is >= lo and f_lo >= want > f_hi.  Pivots are keys strictly above lo, proposed by the lane
// with most keys in range; the workgroup counts the keys >= pivot and narrows the range.  Ends when no key
// lies strictly above lo inside the range: then every key left inside equals lo, the cut value.
// kt is an LDS table [M][threads of the group].
struct Range {
    int a, b;          // this lane's keys inside the range: ks[a..b)
    int f_hi, f_lo;    // keys of the workgroup above the range / above or inside it
    double lo;         // every key inside is >= lo
};
template <int M, bool SINGLE>
__device__ __forceinline__ Range pivot_rounds(const double (&ks)[M], double* kt, int want, Range rg, Group<SINGLE>& g) {
    int a = rg.a, b = rg.b, f_hi = rg.f_hi, f_lo = rg.f_lo;
    double lo = rg.lo;
    const int NT = g.nt, tid = g.tid;
#pragma unroll
    for (int r = 0; r < M; ++r) kt[r * NT + tid] = ks[r];
    // every round moves lo up or the upper end down to a key strictly inside, so M * blockDim rounds
    // always suffice; the bound makes termination unconditional
    for (int round = 0; round < M * 256 + 2; ++round) {
        const int cnt = b - a;
        double prop = nan_d();
        if (cnt > 0) {
            const int T = want - f_hi, R = f_lo - f_hi;
            int q = (int)((float)cnt * (float)(2 * T - 1) * __frcp_rn((float)(2 * R)));
            q = q > cnt - 1 ? cnt - 1 : (q < 0 ? 0 : q);
            const double top = kt[a * NT + tid];
            prop = kt[(a + q) * NT + tid];
            if (!(prop > lo)) prop = top;
        }
        const bool valid = prop > lo;
        const int win = g.max_i(valid ? ((cnt << 16) | (0xffff - tid)) : 0);
        if (win == 0) break;
        const double p = g.bcast(prop, 0xffff - (win & 0xffff));
        int ge = 0;
#pragma unroll
        for (int r = 0; r < M; ++r) ge += ks[r] >= p ? 1 : 0;
        const int f_p = g.sum_i(ge);
        if (f_p >= want) { lo = p; b = ge; f_lo = f_p; }
        else             { a = ge; f_hi = f_p; }
    }
    Range out;
    out.a = a; out.b = b; out.f_hi = f_hi; out.f_lo = f_lo; out.lo = lo;
    return out;
}

// Result of "keep the `want` largest keys of the workgroup".
struct Cut {
    unsigned keep;     // bit r: this lane's key[r] is kept for certain
    double tau;        // every kept key is >= tau, at least `want` keys are >= tau
    int need;          // > 0: besides `keep`, `need` of the `total_eq` keys == tau are kept, in the caller's tie order
    int total_eq;
};

// Every lane holds M keys (NaN = absent); SORTED: in descending order with NaN last.
// kt is an LDS table [M][blockDim] (used only by phase 2), hist an LDS scratch of kBuckets + 4 ints.
//   phase 1  [lo, hi) = [caller's lower bound (or the smallest key), just above the largest key).
//            The keys inside are binned into 256 equal-width buckets (LDS atomics); a suffix scan of
//            the histogram finds the bucket that holds the cut; the same is repeated once inside
//            that bucket (65536 cells overall).  If the cut falls between two cells the kept set is
//            known exactly and the search is over.  Needs no order inside a lane.
//   phase 2  (ties or near-ties at the cut) on sorted keys: pivots are keys strictly inside the
//            remaining range, proposed by the lane with most keys in range; per lane a = #keys
//            above the range, b = #keys above or in it.  Ends when no key lies strictly inside, so
//            that every key left in range equals tau.
template <int M, bool SINGLE, bool SORTED>
__device__ Cut select_keys(const double (&key)[M], double* kt, int* hist, int want, bool have_first,
                           double first_pivot, Group<SINGLE>& g) {
    (void)kt;
    Cut cut;
    cut.keep = 0u; cut.need = 0; cut.total_eq = 0;
    double lmin = nan_d(), lmax = nan_d();
#pragma unroll
    for (int r = 0; r < M; ++r) { lmin = fmin(lmin, key[r]); lmax = fmax(lmax, key[r]); }
    double lo = have_first ? first_pivot : g.min_d(lmin);
    const double gmax = -g.min_d(-lmax);
    unsigned in = 0u;                              // keys inside [lo, hi)
#pragma unroll
    for (int r = 0; r < M; ++r) in |= (key[r] >= lo ? 1u : 0u) << r;
    int f_hi = 0, f_lo = 0;
    bool exact = false;
    if (gmax > lo) {
        const double hi = next_up(gmax);
        double u[M];
        const double scale = (double)kBuckets / (hi - lo);
#pragma unroll
        for (int r = 0; r < M; ++r) u[r] = (key[r] - lo) * scale;
        for (int level = 0; level < 2; ++level) {
            int bk[M];
#pragma unroll
            for (int r = 0; r < M; ++r) {
                int q = (int)u[r];
                bk[r] = q < 0 ? 0 : (q > kBuckets - 1 ? kBuckets - 1 : q);
            }
            // hist is all zero here (cleared once per kernel, and re-cleared by the scan below)
#pragma unroll
            for (int r = 0; r < M; ++r)
                if ((in >> r) & 1u) atomicAdd(&hist[bk[r]], 1);
            lds_sync<SINGLE>();
            const int T = want - f_hi;            // rank of the cut among the keys in range
            int B = -1, above = 0, inb = 0, total = 0;
            if (g.wave == 0) {
                constexpr int BPL = kBuckets / 64;                 // buckets per lane of the scanning wavefront
                const int L = g.lane;
                int c[BPL];
                int sum = 0;
#pragma unroll
                for (int i = 0; i < BPL; ++i) { c[i] = hist[BPL * L + i]; sum += c[i]; }
#pragma unroll
                for (int i = 0; i < BPL; ++i) hist[BPL * L + i] = 0;
                const int P = wave_incl_scan(sum, L);
                total = rl(P, 63);
                const int above_lane = total - P;                 // keys in higher lanes' buckets
                const bool has = above_lane < T && above_lane + sum >= T;
                int Bl = BPL * L, abl = above_lane, inl = 0;
                bool found = false;
#pragma unroll
                for (int i = BPL - 1; i >= 0; --i) {              // highest bucket first
                    if (!found) {
                        if (abl + c[i] >= T) { found = true; Bl = BPL * L + i; inl = c[i]; }
                        else abl += c[i];
                    }
                }
                const u64 bal = __ballot(has);
                if (bal != 0ull) {
                    const int src = __ffsll((long long)bal) - 1;
                    B = rl(Bl, src); above = rl(abl, src); inb = rl(inl, src);
                }
                if (!SINGLE && L == 0) {
                    hist[kBuckets] = B; hist[kBuckets + 1] = above; hist[kBuckets + 2] = inb; hist[kBuckets + 3] = total;
                }
            }
            if (!SINGLE) {
                lds_sync<SINGLE>();
                B = hist[kBuckets]; above = hist[kBuckets + 1]; inb = hist[kBuckets + 2]; total = hist[kBuckets + 3];
            }
            if (level == 0) f_lo = f_hi + total;
            if (B < 0) break;                     // cannot happen while count(key >= lo) >= want; be safe
            unsigned gt = 0u, eq = 0u;
#pragma unroll
            for (int r = 0; r < M; ++r) {
                gt |= (bk[r] > B ? 1u : 0u) << r;
                eq |= (bk[r] == B ? 1u : 0u) << r;
            }
            cut.keep |= in & gt;
            if (above + inb == T) { exact = true; cut.keep |= in & eq; break; }
            in &= eq;
            f_hi += above; f_lo = f_hi + inb;
#pragma unroll
            for (int r = 0; r < M; ++r) u[r] = (u[r] - (double)B) * (double)kBuckets;
        }
    } else {
        f_lo = g.sum_i(__popc(in));
    }
    if (exact) {
        double kmin = nan_d();
#pragma unroll
        for (int r = 0; r < M; ++r) kmin = fmin(kmin, ((cut.keep >> r) & 1u) ? key[r] : nan_d());
        cut.tau = g.min_d(kmin);
        return cut;
    }

    // ---- phase 2 -----------------------------------------------------------------------------
    double ks[M];
#pragma unroll
    for (int r = 0; r < M; ++r) ks[r] = key[r];
    if (!SORTED) sort_desc<M>(ks);
    Range rg;
    rg.a = __popc(cut.keep); rg.b = rg.a + __popc(in); rg.f_hi = f_hi; rg.f_lo = f_lo; rg.lo = lo;
    rg = pivot_rounds<M, SINGLE>(ks, kt, want, rg, g);
    cut.tau = rg.lo;
    cut.keep = 0u;
#pragma unroll
    for (int r = 0; r < M; ++r) cut.keep |= (key[r] > rg.lo ? 1u : 0u) << r;
    cut.need = want - rg.f_hi;
    cut.total_eq = rg.f_lo - rg.f_hi;
    return cut;
}

// One drafting step's cut: how many of this lane's (rank-sorted) candidates survive, and the
// first slot they occupy in the next layer.  tau_out: a value reached by at least `want`
// candidates (NaN when nothing was cut).
template <int KMAX, bool SINGLE>
__device__ void layer_cut(const double (&ck)[KMAX], double* kt, int* hist, bool active, int k, int F, int want,
                          int r0, Group<SINGLE>& g, int& cnt, int& off, double& tau_out) {
    tau_out = nan_d();
    if (k * F <= want) {
        cnt = active ? k : 0;
    } else {
        // every lane holds at least r0+1 candidates and (r0+1) F >= want, so the smallest rank-r0
        // candidate is a lower bound of the cut: it discards most candidates at once
        double c0 = nan_d();
#pragma unroll
        for (int r = 0; r < KMAX; ++r) c0 = (r == r0) ? ck[r] : c0;
        const double m0 = g.min_d(c0);
        const Cut cut = select_keys<KMAX, SINGLE, true>(ck, kt, hist, want, true, m0, g);
        cnt = __popc(cut.keep);               // sorted candidates: the kept ones are a prefix
        if (cut.need > 0) {                   // ties at the cut: smaller parent slot first, then smaller rank
            int lane_eq = 0;
#pragma unroll
            for (int r = 0; r < KMAX; ++r) lane_eq += ck[r] == cut.tau ? 1 : 0;
            int take = lane_eq;
            if (cut.total_eq != cut.need) {
                const int before = g.excl_scan(lane_eq);
                take = cut.need - before;
                take = take < 0 ? 0 : (take > lane_eq ? lane_eq : take);
            }
            cnt += take;
        }
        tau_out = cut.tau;
    }
    off = g.excl_scan(cnt);
}

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

// candidate scores of one frontier slot: log p^(child) = log p^(parent) + (x - lse)   (Eq. 2)
template <int KMAX>
__device__ __forceinline__ void candidate_scores(double S, double lse, const float (&v)[KMAX], bool active, int k,
                                                 double (&ck)[KMAX]) {
#pragma unroll
    for (int r = 0; r < KMAX; ++r)
        ck[r] = (active && r < k) ? S + ((double)v[r] - lse) : __longlong_as_double(0x7ff8000000000000ll);
}

// LDS carve-up shared by the kernels below.  DK = rows of the key region (>= depth, and >= DMAX so
// that the final selection can reuse the region as its key table once the keys sit in registers).
struct Pool {
    double* key;            // [DK][NT]  log p^ of pool node (layer t+1, slot)
    double* kt;             // [KMAX][NT] per-lane key table of the per-step selection
    int* tok;               // [D][NT]
    unsigned char* par;     // [D][NT]   parent slot in the previous layer (< 256)
    unsigned char* oidx;    // [D][NT]   output index of a selected node (< 256)
    u64* mrow;              // [NT][4]   ancestor bitmask rows by output index
};
__device__ __forceinline__ Pool carve_pool(void* smem, int D, int NT, int DK, int KM) {
    Pool p;
    p.key = (double*)smem;
    p.kt = p.key + (size_t)DK * NT;
    p.mrow = (u64*)(p.kt + (size_t)KM * NT);
    p.tok = (int*)(p.mrow + (size_t)NT * 4);
    p.par = (unsigned char*)(p.tok + (size_t)D * NT);
    p.oidx = p.par + (size_t)D * NT;
    return p;
}
inline size_t pool_lds_bytes(int D, int NT, int DK, int KM) {
    return (size_t)DK * NT * 8 + (size_t)KM * NT * 8 + (size_t)NT * 4 * 8 + (size_t)D * NT * (4 + 1 + 1);
}

// Last line of Algorithm 1 and the outputs.  `steps` layers are in the pool; lo0 (or NaN) is a
// value that at least n pool nodes reach (the largest cut value of the steps that cut to n).
// The n best nodes of a pool of `steps` layers (last line of Algorithm 1; also the set whose p^ sum is
// E_sub(T, n)).  pk[t] = log p^ of pool node (layer t+1, slot tid), NaN = absent; lo0 (or NaN) is a value that
// at least n pool nodes reach.  Returns bit t set for the selected nodes of this thread.  Ties at the cut:
// shallower first, then smaller slot.  The pool's key region in LDS becomes the selection's table.
template <int DMAX, bool SINGLE>
__device__ unsigned int pool_select(const SelKArgs& a, const Pool& P, const double (&pk)[DMAX], int steps, int pool_nodes,
                                    double lo0, Group<SINGLE>& g, int* s_hist) {
    const int n = a.n;
    unsigned int sel = 0;           // bit t: pool node (layer t+1, slot tid) is in the tree
    if (pool_nodes <= n) {
#pragma unroll
        for (int t = 0; t < DMAX; ++t) sel |= (pk[t] == pk[t] ? 1u : 0u) << t;
    } else {
        lds_sync<SINGLE>();         // every lane has its pool keys in registers: the key region becomes the table
        const Cut cut = select_keys<DMAX, SINGLE, false>(pk, P.key, s_hist, n, lo0 == lo0, lo0, g);
        sel = cut.keep;
        int need = cut.need;
        if (need > 0 && cut.total_eq == need) {
#pragma unroll
            for (int t = 0; t < DMAX; ++t) sel |= (pk[t] == cut.tau ? 1u : 0u) << t;
        } else if (need > 0) {       // ties at the cut: shallower first, then smaller slot
            for (int t = 0; t < steps; ++t) {
                double kt = nan_d();
#pragma unroll
                for (int tt = 0; tt < DMAX; ++tt) kt = (tt == t) ? pk[tt] : kt;
                const int eq = kt == cut.tau ? 1 : 0;
                const int before = g.excl_scan(eq);
                const int layer_eq = g.sum_i(eq);
                if (eq && before < need) sel |= 1u << t;
                need -= layer_eq < need ? layer_eq : need;
            }
        }
    }
    return sel;
}

template <int DMAX, bool SINGLE>
__device__ void finalize_tree(const SelKArgs& a, const Pool& P, int steps, int b, double lo0, Group<SINGLE>& g,
                              int* s_cntw /*[OT_MAX_DEPTH][4]*/, int* s_hist) {
    const int NT = blockDim.x, tid = threadIdx.x, n = a.n;
    const int W = OT_MASK_WORDS(n);
    int pool_nodes = 0;
    for (int t = 0; t < steps; ++t) pool_nodes += a.F[t + 1];
    const int n_out = pool_nodes < n ? pool_nodes : n;

    double pk[DMAX];
#pragma unroll
    for (int t = 0; t < DMAX; ++t) pk[t] = (t < steps && tid < a.F[t + 1]) ? P.key[t * NT + tid] : nan_d();

    const unsigned int sel = pool_select<DMAX, SINGLE>(a, P, pk, steps, pool_nodes, lo0, g, s_hist);

    // output index = rank in (depth, slot) order among the selected nodes
    const int lane = tid & 63;
    if (SINGLE) {
        int base = 0;               // wave-uniform: nodes selected in shallower layers
#pragma unroll
        for (int t = 0; t < DMAX; ++t) {
            const u64 bal = __ballot((sel >> t) & 1u);
            if ((sel >> t) & 1u) P.oidx[t * NT + tid] = (unsigned char)(base + __popcll(bal & ((1ull << lane) - 1ull)));
            base += __popcll(bal);
        }
    } else {
        int my_prefix[DMAX];
#pragma unroll
        for (int t = 0; t < DMAX; ++t) {
            const u64 bal = __ballot((sel >> t) & 1u);
            my_prefix[t] = __popcll(bal & ((1ull << lane) - 1ull));
            if (lane == 0 && t < steps) s_cntw[t * 4 + g.wave] = __popcll(bal);
        }
        lds_sync<SINGLE>();
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
                if ((sel >> t) & 1u) P.oidx[t * NT + tid] = (unsigned char)(mine + my_prefix[t]);
            }
        }
    }
    lds_sync<SINGLE>();

    // output index of every selected node of this lane and of its parent (independent LDS reads)
    int my_i[DMAX], my_pi[DMAX];
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {
        my_i[t] = 0; my_pi[t] = -1;
        if (t < steps && ((sel >> t) & 1u)) {
            my_i[t] = P.oidx[t * NT + tid];
            if (t > 0) my_pi[t] = P.oidx[(t - 1) * NT + P.par[t * NT + tid]];
        }
    }
    // ancestor masks, layer by layer (a parent's row is complete before its children read it), and
    // the per-node outputs.  The key region is free again: it collects log p^ by output index.
    const size_t ob = (size_t)b * n;
    double* sc_by_index = P.key;
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {
        if (t < steps) {
            if ((sel >> t) & 1u) {
                const int i = my_i[t], pi = my_pi[t];
                u64 row[4] = {0ull, 0ull, 0ull, 0ull};
                if (t > 0) {
#pragma unroll
                    for (int w = 0; w < 4; ++w) row[w] = P.mrow[pi * 4 + w];
                }
#pragma unroll
                for (int w = 0; w < 4; ++w) row[w] |= (w == (i >> 6)) ? (1ull << (i & 63)) : 0ull;
#pragma unroll
                for (int w = 0; w < 4; ++w) P.mrow[i * 4 + w] = row[w];
                sc_by_index[i] = pk[t];
                a.out.token[ob + i] = P.tok[t * NT + tid];
                a.out.parent[ob + i] = pi;
                a.out.depth[ob + i] = t + 1;
                a.out.score[ob + i] = (float)pk[t];
#pragma unroll
                for (int w = 0; w < 4; ++w)
                    if (w < W) a.out.mask[(ob + i) * W + w] = row[w];
            }
            lds_sync<SINGLE>();
        }
    }
    for (int i = n_out + tid; i < n; i += NT) {
        a.out.token[ob + i] = -1;
        a.out.parent[ob + i] = -1;
        a.out.depth[ob + i] = 0;
        a.out.score[ob + i] = -INFINITY;
        for (int w = 0; w < W; ++w) a.out.mask[(ob + i) * W + w] = 0ull;
    }
    // E = sum of p^ (Eq. 3): one exp per lane, node i on lane i
    double e_sum = tid < n_out ? exp(sc_by_index[tid]) : 0.0;
    e_sum = g.sum_d(e_sum);
    if (tid == 0) {
        a.out.expect[b] = e_sum;
        a.out.n_out[b] = n_out;
    }
}

#define OT_SELECT_SHARED                                   \
    extern __shared__ u64 smem[];                          \
    __shared__ int s_red[8];                               \
    __shared__ double s_bc[2];                             \
    __shared__ double s_redd[8];                           \
    __shared__ int s_cntw[OT_MAX_DEPTH * 4];               \
    __shared__ int s_hist[kBuckets + 4];                   \
    Group<SINGLE> g;                                       \
    g.red = s_red; g.bc = s_bc; g.redd = s_redd;           \
    g.phase = g.bphase = g.dphase = 0;                     \
    g.tid = threadIdx.x; g.lane = threadIdx.x & 63;        \
    g.wave = threadIdx.x >> 6; g.nw = blockDim.x >> 6;     \
    g.nt = blockDim.x;                                     \
    for (int i_ = threadIdx.x; i_ < kBuckets + 4; i_ += blockDim.x) s_hist[i_] = 0; \
    __syncthreads();

// One-shot: all steps in one launch, pool resident in LDS.
template <int KMAX, int DMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_oneshot_kernel(const SelKArgs a) {
    OT_SELECT_SHARED
    const int NT = blockDim.x, tid = threadIdx.x, b = blockIdx.x, D = a.depth;
    const Pool P = carve_pool(smem, D, NT, DMAX, KMAX);

    double lse, nlse;
    float v[KMAX], nv[KMAX];
    int id[KMAX], nid[KMAX];
    double lo0 = nan_d();
    load_row<KMAX>(a, (long long)b * a.rows_per_seq + tid, tid < a.F[0], nlse, nv, nid);
    for (int t = 0; t < D; ++t) {
        const int F = a.F[t], Fn = a.F[t + 1];
        const bool active = tid < F;
        lse = nlse;
#pragma unroll
        for (int r = 0; r < KMAX; ++r) { v[r] = nv[r]; id[r] = nid[r]; }
        if (t + 1 < D)   // next step's row: its address does not depend on the tree, fetch it now
            load_row<KMAX>(a, (long long)b * a.rows_per_seq + a.row_start[t + 1] + tid, tid < Fn, nlse, nv, nid);
        const double S = (t == 0 || !active) ? 0.0 : P.key[(t - 1) * NT + tid];
        double ck[KMAX];
        candidate_scores<KMAX>(S, lse, v, active, a.k, ck);
        int cnt, off;
        double tau;
        layer_cut<KMAX, SINGLE>(ck, P.kt, s_hist, active, a.k, F, Fn, a.r0[t], g, cnt, off, tau);
        if (tau == tau) lo0 = (lo0 == lo0) ? fmax(lo0, tau) : tau;
#pragma unroll
        for (int r = 0; r < KMAX; ++r) {
            if (r < cnt) {
                P.key[t * NT + off + r] = ck[r];
                P.tok[t * NT + off + r] = id[r];
                P.par[t * NT + off + r] = (unsigned char)tid;
            }
        }
        lds_sync<SINGLE>();
    }
    finalize_tree<DMAX, SINGLE>(a, P, D, b, lo0, g, s_cntw, s_hist);
}

// Streaming: one drafting step; the pool lives in the caller's workspace between launches.
template <int KMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_step_kernel(const SelKArgs a) {
    if (!a.seq_active[blockIdx.x]) {            // frozen by the adaptive-depth rule: its tree stays as it is
        if (a.frontier_count && threadIdx.x == 0) a.frontier_count[blockIdx.x] = 0;
        return;
    }
    OT_SELECT_SHARED
    (void)s_cntw;
    const int tid = threadIdx.x, b = blockIdx.x, t = a.step, n = a.n;
    const int F = a.F[t], Fn = a.F[t + 1];
    const bool active = tid < F;
    const size_t pb = (size_t)b * a.depth * n;
    double lse;
    float v[KMAX];
    int id[KMAX];
    load_row<KMAX>(a, (long long)b * a.rows_per_seq + tid, active, lse, v, id);
    const double S = (t == 0 || !active) ? 0.0 : a.pool_key[pb + (size_t)(t - 1) * n + tid];
    double ck[KMAX];
    candidate_scores<KMAX>(S, lse, v, active, a.k, ck);
    int cnt, off;
    double tau;
    layer_cut<KMAX, SINGLE>(ck, (double*)smem, s_hist, active, a.k, F, Fn, a.r0[t], g, cnt, off, tau);
    if (tid == 0) {
        a.step_tau[(size_t)b * a.depth + t] = tau;
        a.seq_steps[b] = t + 1;
        if (a.frontier_count) a.frontier_count[b] = Fn;
    }
#pragma unroll
    for (int r = 0; r < KMAX; ++r) {
        if (r < cnt) {
            const size_t o = pb + (size_t)t * n + off + r;
            a.pool_key[o] = ck[r];
            a.pool_p[o] = exp(ck[r]);             // p^ (Eq. 2), kept for E_sub
            a.pool_tok[o] = id[r];
            a.pool_par[o] = tid;
            a.frontier_token[(size_t)b * n + off + r] = id[r];
            a.frontier_parent[(size_t)b * n + off + r] = tid;
        }
    }
    // Root paths of the new frontier over pool indices ((layer t+1, slot s) -> t n + s): the parent's path plus the
    // node itself -- the incremental form of Algorithm 2's mask for the drafting phase.  A path has at most `depth`
    // entries however many nodes the pool holds, so the state stays small; ot_tree_frontier_mask turns it into bits.
    {
        const size_t fa = (size_t)a.gridDim_batch * n * OT_MAX_DEPTH;
        const unsigned short* prev = a.front_anc + (size_t)((t & 1) ^ 1) * fa + ((size_t)b * n + tid) * OT_MAX_DEPTH;
        unsigned short* cur = a.front_anc + (size_t)(t & 1) * fa + (size_t)b * n * OT_MAX_DEPTH;
        for (int r = 0; r < cnt; ++r) {
            unsigned short* row = cur + (size_t)(off + r) * OT_MAX_DEPTH;
            for (int e = 0; e < t; ++e) row[e] = prev[e];
            row[t] = (unsigned short)(t * n + off + r);
        }
    }
}

template <int DMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_finalize_kernel(const SelKArgs a) {
    OT_SELECT_SHARED
    const int NT = blockDim.x, tid = threadIdx.x, b = blockIdx.x, n = a.n;
    const int steps = a.step < a.seq_steps[b] ? a.step : a.seq_steps[b];     // a frozen sequence has fewer layers
    const Pool P = carve_pool(smem, a.depth, NT, DMAX, 0);
    const size_t pb = (size_t)b * a.depth * n;
    double lo0 = nan_d();
    for (int t = 0; t < steps; ++t) {
        if (tid < a.F[t + 1]) {
            const size_t o = pb + (size_t)t * n + tid;
            P.key[t * NT + tid] = a.pool_key[o];
            P.tok[t * NT + tid] = a.pool_tok[o];
            P.par[t * NT + tid] = (unsigned char)a.pool_par[o];
        }
        const double tau = a.step_tau[(size_t)b * a.depth + t];
        if (tau == tau) lo0 = (lo0 == lo0) ? fmax(lo0, tau) : tau;
    }
    __syncthreads();
    finalize_tree<DMAX, SINGLE>(a, P, steps, b, lo0, g, s_cntw, s_hist);
}

// E_sub(T, n) of the tree drafted so far = the sum of the n largest p^ of the pool (Sec. 3, text ahead of
// Algorithm 1), and the loop condition of Algorithm 1: go on while E_sub - E > delta, with E <- E_sub.
// A sequence that stops is frozen (tree_step_kernel skips it, tree_finalize_kernel uses its layer count).
template <int DMAX, bool SINGLE>
__global__ __launch_bounds__(256) void tree_esub_kernel(const SelKArgs a) {
    OT_SELECT_SHARED
    (void)s_cntw;
    const int NT = blockDim.x, tid = threadIdx.x, b = blockIdx.x, n = a.n;
    const int steps = a.step < a.seq_steps[b] ? a.step : a.seq_steps[b];
    const Pool P = carve_pool(smem, a.depth, NT, DMAX, 0);
    const size_t pb = (size_t)b * a.depth * n;
    double lo0 = nan_d();
    int pool_nodes = 0;
    double pk[DMAX], pp[DMAX];
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {
        pk[t] = nan_d(); pp[t] = 0.0;
        if (t < steps) {
            pool_nodes += a.F[t + 1];
            if (tid < a.F[t + 1]) {
                pk[t] = a.pool_key[pb + (size_t)t * n + tid];
                pp[t] = a.pool_p[pb + (size_t)t * n + tid];
            }
            const double tau = a.step_tau[(size_t)b * a.depth + t];
            if (tau == tau) lo0 = (lo0 == lo0) ? fmax(lo0, tau) : tau;
        }
    }
    __syncthreads();
    const unsigned int sel = pool_select<DMAX, SINGLE>(a, P, pk, steps, pool_nodes, lo0, g, s_hist);
    double e = 0.0;
#pragma unroll
    for (int t = 0; t < DMAX; ++t) e += ((sel >> t) & 1u) ? pp[t] : 0.0;
    e = g.sum_d(e);
    if (tid == 0) {
        a.e_sub[b] = e;
        int go = 0;
        if (a.seq_active[b]) {
            go = (e - a.seq_E[b] > a.delta) ? 1 : 0;
            if (go) a.seq_E[b] = e; else a.seq_active[b] = 0;
        }
        a.go_on[b] = go;
    }
}

// The frontier's ancestor masks, from the root paths the step kernel keeps: mask_out [batch][n][mask_words]
__global__ __launch_bounds__(256) void tree_front_mask_kernel(const SelKArgs a) {
    const int b = blockIdx.x, n = a.n;
    const int steps = a.step < a.seq_steps[b] ? a.step : a.seq_steps[b];
    const int F = steps > 0 ? a.F[steps] : 0;
    const size_t fa = (size_t)a.gridDim_batch * n * OT_MAX_DEPTH;
    const unsigned short* src = a.front_anc + (size_t)((steps - 1) & 1) * fa + (size_t)b * n * OT_MAX_DEPTH;
    for (int i = threadIdx.x; i < n * a.mask_words; i += blockDim.x) {
        const int s = i / a.mask_words, w = i - s * a.mask_words;
        u64 bits = 0ull;
        if (s < F)
            for (int e = 0; e < steps; ++e) {
                const int idx = src[(size_t)s * OT_MAX_DEPTH + e];
                if ((idx >> 6) == w) bits |= 1ull << (idx & 63);
            }
        a.mask_out[(size_t)b * n * a.mask_words + i] = bits;
    }
}

__global__ void tree_begin_kernel(double* seq_E, int32_t* seq_steps, int32_t* seq_active, int batch) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) { seq_E[b] = 0.0; seq_steps[b] = 0; seq_active[b] = 1; }
}

// ---------------------------------------------------------------------------
// Fast path: n <= 64 (one wavefront owns the whole frontier, no barriers after the prologue) and the
// row statistics of the whole tree fit in LDS.
//   prologue  256 threads turn (top-k logits, lse) of every row into log-probabilities
//             dl[row][r] = x - lse (fp64) in LDS; three of the four wavefronts then leave.
//   step t    lane j: ck[r] = S_j + dl[row(t, j)][r] -- already sorted by rank; cut_sorted() finds how
//             many of them survive; only (log p^, parent slot, rank) go to the pool, token ids are
//             fetched at the end, for the nodes of the tree only.
//   finish    final selection, then every tree node moves to the lane of its output index: the
//             ancestor masks (one 64-bit word) are built with lane permutes by pointer doubling
//             and all outputs are written with one store each.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double wave_max_d(double v) {
    v = fmax(v, dpp_d<DPP_QUAD_XOR1>(v));
    v = fmax(v, dpp_d<DPP_QUAD_XOR2>(v));
    v = fmax(v, dpp_d<DPP_ROW_HALF_MIRROR>(v));
    v = fmax(v, dpp_d<DPP_ROW_MIRROR>(v));
    return fmax(fmax(rl_d(v, 0), rl_d(v, 16)), fmax(rl_d(v, 32), rl_d(v, 48)));
}

// Bounds of a bracket do not have to be tight, only safe: a value not above the smallest (not below the
// largest) of the lanes' doubles, from an fp32 reduction (one DPP instruction per stage) widened by more
// than the conversion error.  NaN lanes are ignored; all NaN gives NaN.
__device__ __forceinline__ double wave_lower_bound(double v) {
    float f = (float)v;
    f = fminf(f, __int_as_float(dpp_i<DPP_QUAD_XOR1>(__float_as_int(f), __float_as_int(f))));
    f = fminf(f, __int_as_float(dpp_i<DPP_QUAD_XOR2>(__float_as_int(f), __float_as_int(f))));
    f = fminf(f, __int_as_float(dpp_i<DPP_ROW_HALF_MIRROR>(__float_as_int(f), __float_as_int(f))));
    f = fminf(f, __int_as_float(dpp_i<DPP_ROW_MIRROR>(__float_as_int(f), __float_as_int(f))));
    const float m = fminf(fminf(rl_f(f, 0), rl_f(f, 16)), fminf(rl_f(f, 32), rl_f(f, 48)));
    return (double)m - (fabs((double)m) * 1.2e-7 + 1e-30);
}
__device__ __forceinline__ double wave_upper_bound(double v) {
    const float m = wave_max_f((float)v);
    return (double)m + (fabs((double)m) * 1.2e-7 + 1e-30);
}

// The cut bucket of a 256-bin histogram (one wavefront; lane L scans bins 4L..4L+3 and clears them):
// B = the bin that holds the T-th largest key, above = keys in higher bins, inb = keys in bin B,
// total = all keys.  B = -1 if there are fewer than T keys.
__device__ __forceinline__ void hist_cut(int* hist, int T, int L, int& B, int& above, int& inb, int& total) {
    constexpr int BPL = kBuckets / 64;
    int c[BPL];
    int sum = 0;
#pragma unroll
    for (int i = 0; i < BPL; ++i) { c[i] = hist[BPL * L + i]; sum += c[i]; }
#pragma unroll
    for (int i = 0; i < BPL; ++i) hist[BPL * L + i] = 0;
    const int P = wave_incl_scan(sum, L);
    total = rl(P, 63);
    const int above_lane = total - P;                 // keys in higher lanes' bins
    const bool has = above_lane < T && above_lane + sum >= T;
    int Bl = BPL * L, abl = above_lane, inl = 0;
    bool found = false;
#pragma unroll
    for (int i = BPL - 1; i >= 0; --i) {              // highest bin first
        if (!found) {
            if (abl + c[i] >= T) { found = true; Bl = BPL * L + i; inl = c[i]; }
            else abl += c[i];
        }
    }
    const u64 bal = __ballot(has);
    B = -1; above = 0; inb = 0;
    if (bal != 0ull) {
        const int src = __ffsll((long long)bal) - 1;
        B = rl(Bl, src); above = rl(abl, src); inb = rl(inl, src);
    }
}

// "Keep the `want` largest of the wavefront's keys" for keys that are sorted inside every lane.
// ck: this lane's keys, descending, NaN = absent (NaN last).  lo: at least `want` keys are >= lo.
// Result: exact = true: the cnt largest keys of this lane are kept (all kept keys are strictly larger
// than all others).  exact = false: the keys > tau are kept (cnt of this lane's), and `need` of the
// `total_eq` keys == tau, in an order the caller defines.
// The survivors of a lane are a prefix of its list, so the search keeps two prefix lengths per lane,
// a (certainly kept) <= b (kept or undecided), instead of per-key flags:
//   two histogram levels (256 bins each) over [lower bound, largest key] narrow the undecided keys to
//   one of 65536 cells; if the cut falls between two bins the answer is exact and the search is over,
//   otherwise the pivot rounds finish on the few keys left.
struct SortedCut {
    int cnt;
    bool exact;
    double tau;
    int need, total_eq;
};
template <int M>
__device__ __forceinline__ SortedCut cut_sorted(const double (&ck)[M], double* kt, int* hist, int want, double lo,
                                                int lane, Group<true>& g) {
    SortedCut out;
    out.exact = false; out.tau = lo; out.need = 0; out.total_eq = 0;
    const double gmax = wave_upper_bound(ck[0]);       // only the bracket's upper end: need not be a key
    int a = 0, b = 0;
#pragma unroll
    for (int r = 0; r < M; ++r) b += ck[r] >= lo ? 1 : 0;
    int f_hi = 0, f_lo = 0;
    if (gmax > lo) {
        // u = (key - lo) * scale lies in [0, 256) for every key in [lo, gmax]; the factor below 256 absorbs
        // the error of the approximate reciprocal.  Keys below lo or absent give u <= 0 or NaN -> bin 0,
        // and are kept out by the prefix length b.
        const double scale = 255.9 * __builtin_amdgcn_rcp(gmax - lo);
        double u[M];
#pragma unroll
        for (int r = 0; r < M; ++r) u[r] = (ck[r] - lo) * scale;
        for (int level = 0; level < 2; ++level) {
            int bk[M];
#pragma unroll
            for (int r = 0; r < M; ++r) {
                const int q = (int)u[r];              // saturating; NaN -> 0
                bk[r] = q < 0 ? 0 : q;                // keys above the range (level 1) keep a value >= 256
            }
#pragma unroll
            for (int r = 0; r < M; ++r)
                if (r >= a && r < b) atomicAdd(&hist[bk[r]], 1);
            lds_sync<true>();
            const int T = want - f_hi;                // rank of the cut among the undecided keys
            int B, above, inb, total;
            hist_cut(hist, T, lane, B, above, inb, total);
            if (level == 0) f_lo = total;
            if (B < 0) break;                         // cannot happen (at least `want` keys are >= lo); be safe
            int n_gt = 0, n_ge = 0;                   // prefix lengths: keys above bin B, keys in or above it
#pragma unroll
            for (int r = 0; r < M; ++r) { n_gt += bk[r] > B ? 1 : 0; n_ge += bk[r] >= B ? 1 : 0; }
            n_ge = n_ge < b ? n_ge : b;               // bin 0 also collects the keys below the range
            n_gt = n_gt < b ? n_gt : b;
            if (above + inb == T) {                   // the cut falls between two bins
                out.cnt = n_ge; out.exact = true;
                return out;
            }
            a = n_gt; b = n_ge;
            f_hi += above; f_lo = f_hi + inb;
#pragma unroll
            for (int r = 0; r < M; ++r) u[r] = (u[r] - (double)B) * (double)kBuckets;
        }
    } else {
        f_lo = wave_sum_u(b);                          // every key >= lo equals lo
    }
    Range rg;
    rg.a = a; rg.b = b; rg.f_hi = f_hi; rg.f_lo = f_lo; rg.lo = lo;
    rg = pivot_rounds<M, true>(ck, kt, want, rg, g);
    int cnt = 0;
#pragma unroll
    for (int r = 0; r < M; ++r) cnt += ck[r] > rg.lo ? 1 : 0;
    out.cnt = cnt; out.tau = rg.lo; out.need = want - rg.f_hi; out.total_eq = rg.f_lo - rg.f_hi;
    return out;
}

// One drafting step: how many of this lane's candidates (sorted by rank) survive the cut to `want`.
// r0: every lane that has candidates has more than r0 of them and (r0 + 1) x (such lanes) >= want, so the
// smallest rank-r0 candidate is a lower bound of the cut.  Ties at the cut go to the smaller lane
// (parent slot), then the smaller rank.
template <int M>
__device__ __forceinline__ int step_cut(const double (&ck)[M], double* kt, int* hist, int want, int r0, int lane,
                                        Group<true>& g) {
    double c0 = ck[0];
    if (r0 != 0) {
#pragma unroll
        for (int r = 1; r < M; ++r) c0 = (r == r0) ? ck[r] : c0;
    }
    const SortedCut sc = cut_sorted<M>(ck, kt, hist, want, wave_lower_bound(c0), lane, g);
    if (sc.exact) return sc.cnt;
    int lane_eq = 0;
#pragma unroll
    for (int r = 0; r < M; ++r) lane_eq += ck[r] == sc.tau ? 1 : 0;
    int take = lane_eq;
    if (sc.total_eq != sc.need) {
        const int before = wave_incl_scan(lane_eq, lane) - lane_eq;
        take = sc.need - before;
        take = take < 0 ? 0 : (take > lane_eq ? lane_eq : take);
    }
    return sc.cnt + take;
}

struct FastLds {
    double* dl;               // [rows + 1][KMAX]  log-probabilities of the top-k of every row; last row: NaN
    double* key;              // [DMAX][64]        pool: log p^ by (layer, slot); later the final selection's table
    double* kt;               // [KMAX][64]        table of the pivot rounds; later the nodes by output index
    unsigned short* meta;     // [DMAX][64]        pool: parent slot | rank << 8
    unsigned char* oidx;      // [DMAX][64]        output index of a selected pool node
};
// pool keys, key table, meta, output indices: the part of the LDS layout the final selection works on
__host__ __device__ inline size_t fast_pool_bytes(int KMAX, int DMAX) {
    const int km = KMAX < 4 ? 4 : KMAX;               // the table doubles as 64 x 16 bytes of node records
    return (size_t)DMAX * 64 * 8 + (size_t)km * 64 * 8 + (size_t)DMAX * 64 * 2 + (size_t)DMAX * 64;
}
// rehearse: a second copy of the pool part for the wavefront that rehearses the final selection
__host__ __device__ inline size_t fast_lds_bytes(int rows, int KMAX, int DMAX, bool rehearse) {
    return (size_t)(rows + 1) * KMAX * 8 + fast_pool_bytes(KMAX, DMAX) * (rehearse ? 2 : 1);
}

// p^ = e^key for key <= 0, to about 1e-7 relative: fp32 exp2 of the leading part of key * log2(e), first-order
// correction for the remainder (an fp64 exp costs an order of magnitude more instructions)
__device__ __forceinline__ double exp_of_logp(double key) {
    const double t = key * 1.4426950408889634;
    const float hi = (float)t;
    const double lo = t - (double)hi;
    return (double)__builtin_amdgcn_exp2f(hi) * (1.0 + lo * 0.6931471805599453);
}

// ADAPT: Algorithm 1 with its stopping rule inside the kernel.  The n best nodes drafted so far are kept as a
// running set, one (log p^, p^) per lane; after every step the new layer is merged into it (top n of at most
// 2n keys, two per lane), E_sub(T, n) is the sum of its p^, and drafting stops when E_sub - E <= delta.
template <int KMAX, int DMAX, bool ADAPT>
// The leading scalar arguments repeat fields of `a`: they are what the prologue's loads need, and as separate
// arguments the hardware hands them over in registers at wavefront start (kernel-argument preload), so the loads
// go out without waiting for a read of the argument block.
__global__ __launch_bounds__(256) void tree_fast_kernel(const float* row_topv, const double* row_lse, const int k,
                                                        const int rows, const SelKArgs a) {
    extern __shared__ __attribute__((aligned(16))) u64 smem[];
    __shared__ int s_hist2[2][kBuckets + 4];
    const int tid = threadIdx.x, b = blockIdx.x, n = a.n;
    int D = a.depth;                                  // ADAPT: becomes the number of steps drafted
    FastLds P;
    P.dl = (double*)smem;
    P.key = P.dl + (size_t)(rows + 1) * KMAX;
    P.kt = P.key + DMAX * 64;
    P.meta = (unsigned short*)(P.kt + (KMAX < 4 ? 4 : KMAX) * 64);
    P.oidx = (unsigned char*)(P.meta + DMAX * 64);
    const size_t rbase = (size_t)b * rows;

    // ---- prologue, all four wavefronts ----
    for (int i = tid; i < 2 * (kBuckets + 4); i += 256) (&s_hist2[0][0])[i] = 0;
    // one row per thread and pass: lse once, the k logits of the row, k subtractions; row `rows` is all NaN.  The
    // loads of two passes go out together and unconditionally (indices clamped to valid entries, results
    // discarded where they do not apply): each trip to memory costs more than the arithmetic of a pass.
    {
        const float* tv = row_topv + rbase * k;
        const double* tl = row_lse + rbase;
        for (int row0 = tid; row0 <= rows; row0 += 512) {
            float x[2][KMAX];
            double lse[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int rc = min(row0 + 256 * u, rows - 1);
                lse[u] = tl[rc];
#pragma unroll
                for (int r = 0; r < KMAX; ++r) x[u][r] = tv[rc * k + min(r, k - 1)];
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int row = row0 + 256 * u;
                if (row <= rows) {
                    const bool real = row < rows;
#pragma unroll
                    for (int r = 0; r < KMAX; r += 2) {
                        double2 d2;                   // log p = x - lse (Eq. 2, log space); NaN = absent
                        d2.x = (real && r < k) ? (double)x[u][r] - lse[u] : nan_d();
                        d2.y = (real && r + 1 < k) ? (double)x[u][r + 1] - lse[u] : nan_d();
                        *(double2*)(P.dl + (size_t)row * KMAX + r) = d2;
                    }
                }
            }
        }
    }
    __syncthreads();
    // Wavefront 0 builds the tree.  The kernel's one workgroup lands on a different compute unit from launch to
    // launch, and the first pass through the final selection then waits about 2 us for its instructions.  So while
    // wavefront 0 is drafting, wavefront 1 rehearses the final selection once on made-up keys in an LDS region of
    // its own: the same instructions, no global memory access, results discarded.  (Rehearsing a drafting step in
    // a third wavefront was tried: wavefront 0 reaches that code too soon for it to help.)
    const bool live = __builtin_amdgcn_readfirstlane(tid) < 64;
    if (tid >= (a.rehearse ? 128 : 64)) return;
    const int lane = tid & 63;
    int* const s_hist = s_hist2[live ? 0 : 1];
    if (!live) {
        char* sh = (char*)smem + (size_t)(rows + 1) * KMAX * 8 + fast_pool_bytes(KMAX, DMAX);
        P.key = (double*)sh;
        P.kt = P.key + DMAX * 64;
        P.meta = (unsigned short*)(P.kt + (KMAX < 4 ? 4 : KMAX) * 64);
        P.oidx = (unsigned char*)(P.meta + DMAX * 64);
#pragma unroll
        for (int t = 0; t < DMAX; ++t) {              // distinct keys, every node a first child of the slot above it
            P.key[t * 64 + lane] = -0.5 - 0.01 * (double)(t * 64 + lane);
            P.meta[t * 64 + lane] = (unsigned short)lane;
        }
        lds_sync<true>();
    }
    Group<true> g;
    g.red = nullptr; g.bc = nullptr; g.redd = nullptr;
    g.phase = g.bphase = g.dphase = 0;
    g.tid = lane; g.lane = lane; g.wave = 0; g.nw = 1; g.nt = 64;

    double run_key = nan_d(), run_p = 0.0;            // ADAPT: this lane's member of the running top-n set
    double E_prev = 0.0, E_sub = 0.0;                 // ADAPT: E of Algorithm 1's loop, latest E_sub(T, n)
    // ---- Algorithm 1, step by step ----
    for (int t = 0; live && t < D; ++t) {
        const int F = a.F[t], Fn = a.F[t + 1];
        const bool active = lane < F;
        const double* drow = P.dl + (size_t)(active ? a.row_start[t] + lane : rows) * KMAX;
        const double S = t == 0 ? 0.0 : P.key[(t - 1) * 64 + lane];
        double ck[KMAX];
#pragma unroll
        for (int r = 0; r < KMAX; r += 2) {
            const double2 d2 = *(const double2*)(drow + r);
            ck[r] = S + d2.x;                         // log p^(child) = log p^(parent) + log p   (Eq. 2)
            ck[r + 1] = S + d2.y;
        }
        int cnt;
        if (k * F <= Fn) cnt = active ? k : 0;
        else cnt = step_cut<KMAX>(ck, P.kt, s_hist, Fn, a.r0[t], lane, g);
        const int off = wave_incl_scan(cnt, lane) - cnt;
#pragma unroll
        for (int r = 0; r < KMAX; ++r) {
            if (r < cnt) {
                P.key[t * 64 + off + r] = ck[r];
                P.meta[t * 64 + off + r] = (unsigned short)(lane | (r << 8));
            }
        }
        lds_sync<true>();
        if (ADAPT) {
            // merge the new layer (slot `lane`, if any) into the running set: this lane's pair, larger key first
            const bool has_new = lane < Fn;
            const double nkey = has_new ? P.key[t * 64 + lane] : nan_d();
            const double np = has_new ? exp_of_logp(nkey) : 0.0;
            const bool new_first = (nkey == nkey) && !(run_key >= nkey);
            double pr[2], pp[2];
            pr[0] = new_first ? nkey : run_key; pp[0] = new_first ? np : run_p;
            pr[1] = new_first ? run_key : nkey; pp[1] = new_first ? run_p : np;
            const int have = (pr[0] == pr[0] ? 1 : 0) + (pr[1] == pr[1] ? 1 : 0);
            const int total = wave_sum_u(have);
            int keep = have;
            if (total > n) {
                const SortedCut sc = cut_sorted<2>(pr, P.kt, s_hist, n, wave_lower_bound(fmin(pr[0], pr[1])), lane, g);
                keep = sc.cnt;
                if (!sc.exact) {                      // equal keys at the cut: equal p^, any of them will do (lane order)
                    int lane_eq = (pr[0] == sc.tau ? 1 : 0) + (pr[1] == sc.tau ? 1 : 0);
                    int take = lane_eq;
                    if (sc.total_eq != sc.need) {
                        const int before = wave_incl_scan(lane_eq, lane) - lane_eq;
                        take = sc.need - before;
                        take = take < 0 ? 0 : (take > lane_eq ? lane_eq : take);
                    }
                    keep += take;
                }
            }
            E_sub = wave_sum_d((keep > 0 ? pp[0] : 0.0) + (keep > 1 ? pp[1] : 0.0));
            // back to one member per lane
            const int koff = wave_incl_scan(keep, lane) - keep;
            double* rec = P.kt;                       // [64][2]: (log p^, p^)
            if (keep > 0) { rec[2 * koff] = pr[0]; rec[2 * koff + 1] = pp[0]; }
            if (keep > 1) { rec[2 * koff + 2] = pr[1]; rec[2 * koff + 3] = pp[1]; }
            lds_sync<true>();
            const bool mine = lane < (total < n ? total : n);
            run_key = mine ? rec[2 * lane] : nan_d();
            run_p = mine ? rec[2 * lane + 1] : 0.0;
            lds_sync<true>();
            // the loop condition of Algorithm 1: another step only while the gain of the last one exceeds delta
            if (t + 1 < D) {
                if (!(E_sub - E_prev > a.delta)) { D = t + 1; break; }
                E_prev = E_sub;
            }
        }
    }
    if (ADAPT && live && lane == 0) { a.steps_used[b] = D; a.e_sub[b] = E_sub; }

    // ---- last line of Algorithm 1: the n best nodes of the pool ----
    int pool_nodes = 0;
    for (int t = 0; t < D; ++t) pool_nodes += a.F[t + 1];
    const int n_out = pool_nodes < n ? pool_nodes : n;
    double pk[DMAX];
    int tk[DMAX], mt[DMAX];
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {
        const bool valid = t < D && lane < a.F[t + 1];
        pk[t] = valid ? P.key[t * 64 + lane] : nan_d();
        mt[t] = valid ? (int)P.meta[t * 64 + lane] : 0;
    }
    const int32_t* ti = a.row_topi + rbase * k;
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {                  // token ids: in flight during the selection
        tk[t] = 0;
        if (live && t < D && lane < a.F[t + 1]) tk[t] = ti[(a.row_start[t] + (mt[t] & 255)) * k + (mt[t] >> 8)];
    }
    unsigned int sel = 0;                             // bit t: pool node (layer t+1, slot lane) is in the tree
    if (pool_nodes <= n) {
#pragma unroll
        for (int t = 0; t < DMAX; ++t) sel |= (pk[t] == pk[t] ? 1u : 0u) << t;
    } else {
        // lower bound of the cut: a layer with n nodes -- at least n pool nodes reach its smallest log p^;
        // failing that, the smallest log p^ of the pool
        double lo0 = nan_d();
        int used = 0;
#pragma unroll
        for (int t = 0; t < DMAX; ++t)
            if (t < D && a.F[t + 1] >= n && used < 2) { lo0 = fmax(lo0, wave_lower_bound(pk[t])); ++used; }
        if (used == 0) {
            double lmin = nan_d();
#pragma unroll
            for (int t = 0; t < DMAX; ++t) lmin = fmin(lmin, pk[t]);
            lo0 = wave_lower_bound(lmin);
        }
        // Quick search on the unsorted keys: every key >= lo0 gets a 16-bit code, monotone in the key, over
        // [lo0, largest key]; a 256-bin histogram of the high byte finds the bin of the cut, if needed a second
        // one of the low byte inside that bin.  When the cut falls between two codes the tree is "code >= cut
        // code"; otherwise (ties or near-ties at the cut) the exact search below decides.
        bool done = false;
        {
            double lmax = nan_d();
#pragma unroll
            for (int t = 0; t < DMAX; ++t) lmax = fmax(lmax, pk[t]);
            const double gmax = wave_upper_bound(lmax);
            if (gmax > lo0) {
                const double scale = 65535.0 * __builtin_amdgcn_rcp(gmax - lo0);
                int code[DMAX];
#pragma unroll
                for (int t = 0; t < DMAX; ++t) {
                    const int q = (int)((pk[t] - lo0) * scale);          // saturating; NaN -> 0
                    code[t] = pk[t] >= lo0 ? (q > 65535 ? 65535 : q) : -1;    // -1: below the bound or absent
                }
#pragma unroll
                for (int t = 0; t < DMAX; ++t)
                    if (code[t] >= 0) atomicAdd(&s_hist[code[t] >> 8], 1);
                lds_sync<true>();
                int B0, above0, inb0, total0;
                hist_cut(s_hist, n, lane, B0, above0, inb0, total0);
                if (B0 >= 0) {
                    int cut_code = -1;
                    if (above0 + inb0 == n) {
                        cut_code = B0 << 8;
                    } else {
#pragma unroll
                        for (int t = 0; t < DMAX; ++t)
                            if ((code[t] >> 8) == B0) atomicAdd(&s_hist[code[t] & 255], 1);
                        lds_sync<true>();
                        int B1, above1, inb1, total1;
                        hist_cut(s_hist, n - above0, lane, B1, above1, inb1, total1);
                        if (B1 >= 0 && above1 + inb1 == n - above0) cut_code = (B0 << 8) | B1;
                    }
                    if (cut_code >= 0) {
#pragma unroll
                        for (int t = 0; t < DMAX; ++t) sel |= (code[t] >= cut_code ? 1u : 0u) << t;
                        done = true;
                    }
                }
            }
        }
        if (!done) {
        // exact search: the lane's pool keys, sorted, go through the same routine as a drafting step
        double ps[DMAX];
#pragma unroll
        for (int t = 0; t < DMAX; ++t) ps[t] = pk[t];
        sort_desc<DMAX>(ps);
        lds_sync<true>();                             // the pool keys sit in registers: their LDS region becomes the table
        const SortedCut sc = cut_sorted<DMAX>(ps, P.key, s_hist, n, lo0, lane, g);
        if (sc.exact) {
            double thr = nan_d();                     // this lane's smallest kept key
#pragma unroll
            for (int t = 0; t < DMAX; ++t) thr = (t == sc.cnt - 1) ? ps[t] : thr;
#pragma unroll
            for (int t = 0; t < DMAX; ++t) sel |= (pk[t] >= thr ? 1u : 0u) << t;      // thr = NaN: none
        } else {
#pragma unroll
            for (int t = 0; t < DMAX; ++t) sel |= (pk[t] > sc.tau ? 1u : 0u) << t;
            int need = sc.need;
            if (need > 0 && sc.total_eq == need) {
#pragma unroll
                for (int t = 0; t < DMAX; ++t) sel |= (pk[t] == sc.tau ? 1u : 0u) << t;
            } else if (need > 0) {                    // ties at the cut: shallower first, then smaller slot
#pragma unroll
                for (int t = 0; t < DMAX; ++t) {
                    if (t < D) {
                        const u64 bal = __ballot(pk[t] == sc.tau);
                        const int before = __popcll(bal & ((1ull << lane) - 1ull));
                        if (pk[t] == sc.tau && before < need) sel |= 1u << t;
                        const int layer_eq = __popcll(bal);
                        need -= layer_eq < need ? layer_eq : need;
                    }
                }
            }
        }
        }
    }

    // output index = rank in (depth, slot) order among the selected nodes
    int my_i[DMAX];
    {
        int base = 0;
#pragma unroll
        for (int t = 0; t < DMAX; ++t) {
            const u64 bal = __ballot((sel >> t) & 1u);
            my_i[t] = base + __popcll(bal & ((1ull << lane) - 1ull));
            if ((sel >> t) & 1u) P.oidx[t * 64 + lane] = (unsigned char)my_i[t];
            base += __popcll(bal);
        }
    }
    lds_sync<true>();
    // every tree node moves to the lane of its output index: 16-byte record (log p^, token, parent | depth << 16)
    u64* rec = (u64*)P.kt;
#pragma unroll
    for (int t = 0; t < DMAX; ++t) {
        if ((sel >> t) & 1u) {
            const int pi = t > 0 ? (int)P.oidx[(t - 1) * 64 + (mt[t] & 255)] : 0xffff;
            rec[2 * my_i[t]] = (u64)__double_as_longlong(pk[t]);
            rec[2 * my_i[t] + 1] = (u64)(unsigned)tk[t] | ((u64)(unsigned)(pi | ((t + 1) << 16)) << 32);
        }
    }
    lds_sync<true>();
    const bool node = lane < n_out;
    double key = nan_d();
    int tok = -1, par = -1, dep = 0;
    if (node) {
        key = __longlong_as_double((long long)rec[2 * lane]);
        const u64 w = rec[2 * lane + 1];
        tok = (int)(unsigned)w;
        const unsigned pd = (unsigned)(w >> 32);
        par = (pd & 0xffff) == 0xffff ? -1 : (int)(pd & 0xffff);
        dep = (int)(pd >> 16);
    }
    // ancestor masks (Algorithm 2) by pointer doubling: after round r, m covers the node and its 2^(r+1) - 1
    // nearest ancestors, anc is the 2^(r+1)-th ancestor (a depth-1 node stands for "none": it points at itself)
    u64 m = node ? 1ull << lane : 0ull;
    int anc = (node && par >= 0) ? par : lane;
    for (int span = 1; span < D; span *= 2) {
        const unsigned lo32 = (unsigned)__shfl((int)(unsigned)m, anc);
        const unsigned hi32 = (unsigned)__shfl((int)(unsigned)(m >> 32), anc);
        m |= (u64)lo32 | ((u64)hi32 << 32);
        anc = __shfl(anc, anc);
    }
    if (live && lane < n) {
        const size_t o = (size_t)b * n + lane;
        a.out.token[o] = tok;
        a.out.parent[o] = par;
        a.out.depth[o] = dep;
        a.out.score[o] = node ? (float)key : -INFINITY;
        a.out.mask[o] = m;                            // n <= 64: one mask word per node
    }
    // E = sum of p^ (Eq. 3)
    const double e_sum = wave_sum_d(node ? exp_of_logp(key) : 0.0);
    if (live && lane == 0) {
        a.out.expect[b] = e_sum;
        a.out.n_out[b] = n_out;
    }
}

SelKArgs make_args(const SelectGeometry& g, const BuildWorkspace& ws) {
    SelKArgs a;
    a.row_lse = ws.row_lse; a.row_topv = ws.row_topv; a.row_topi = ws.row_topi;
    a.k = g.k; a.n = g.n; a.depth = g.depth; a.rows_per_seq = g.rows_per_seq;
    for (int i = 0; i < OT_MAX_DEPTH + 2; ++i) {
        a.F[i] = g.F[i];
        a.row_start[i] = g.row_start[i];
        a.r0[i] = 0;
    }
    for (int t = 0; t < g.depth; ++t) {
        const int want = g.F[t + 1], F = g.F[t];
        a.r0[t] = F > 0 ? (want + F - 1) / F - 1 : 0;
    }
    a.pool_key = ws.pool_key; a.pool_tok = ws.pool_tok; a.pool_par = ws.pool_par; a.step_tau = ws.step_tau;
    a.pool_p = ws.pool_p; a.seq_E = ws.seq_E; a.seq_steps = ws.seq_steps; a.seq_active = ws.seq_active;
    a.e_sub = nullptr; a.go_on = nullptr; a.delta = 0.0;
    a.steps_used = nullptr;
    a.front_anc = ws.front_anc; a.mask_out = nullptr; a.mask_words = 0; a.gridDim_batch = g.batch;
    a.out = ot_tree_out{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    a.frontier_token = nullptr; a.frontier_parent = nullptr; a.frontier_count = nullptr;
    a.step = 0;
    a.rehearse = 0;
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
int launch_oneshot_t(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    const size_t lds = pool_lds_bytes(a.depth, NT, DMAX, KMAX);
    int st = set_lds(tree_oneshot_kernel<KMAX, DMAX, SINGLE>, lds);
    if (st != OT_OK) return st;
    hipLaunchKernelGGL((tree_oneshot_kernel<KMAX, DMAX, SINGLE>), dim3(batch), dim3(NT), lds, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}
template <int KMAX, bool SINGLE>
int launch_oneshot_k(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    if (a.depth <= 8) return launch_oneshot_t<KMAX, 8, SINGLE>(a, batch, NT, s);
    if (a.depth <= 10) return launch_oneshot_t<KMAX, 10, SINGLE>(a, batch, NT, s);
    if (a.depth <= 12) return launch_oneshot_t<KMAX, 12, SINGLE>(a, batch, NT, s);
    if (a.depth <= 16) return launch_oneshot_t<KMAX, 16, SINGLE>(a, batch, NT, s);
    if (a.depth <= 20) return launch_oneshot_t<KMAX, 20, SINGLE>(a, batch, NT, s);
    return launch_oneshot_t<KMAX, 32, SINGLE>(a, batch, NT, s);
}
template <bool SINGLE>
int launch_oneshot_s(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    if (a.k <= 4) return launch_oneshot_k<4, SINGLE>(a, batch, NT, s);
    if (a.k <= 8) return launch_oneshot_k<8, SINGLE>(a, batch, NT, s);
    if (a.k <= 10) return launch_oneshot_k<10, SINGLE>(a, batch, NT, s);
    return launch_oneshot_k<16, SINGLE>(a, batch, NT, s);
}

template <int KMAX, bool SINGLE>
int launch_step_t(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    const size_t lds = (size_t)KMAX * NT * 8;
    hipLaunchKernelGGL((tree_step_kernel<KMAX, SINGLE>), dim3(batch), dim3(NT), lds, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}
template <bool SINGLE>
int launch_step_s(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    if (a.k <= 4) return launch_step_t<4, SINGLE>(a, batch, NT, s);
    if (a.k <= 8) return launch_step_t<8, SINGLE>(a, batch, NT, s);
    if (a.k <= 10) return launch_step_t<10, SINGLE>(a, batch, NT, s);
    return launch_step_t<16, SINGLE>(a, batch, NT, s);
}

template <int DMAX, bool SINGLE>
int launch_finalize_t(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    const size_t lds = pool_lds_bytes(a.depth, NT, DMAX, 0);
    int st = set_lds(tree_finalize_kernel<DMAX, SINGLE>, lds);
    if (st != OT_OK) return st;
    hipLaunchKernelGGL((tree_finalize_kernel<DMAX, SINGLE>), dim3(batch), dim3(NT), lds, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

// LDS the fast path may use (of the 160 KB of a compute unit)
constexpr size_t kFastLdsLimit = 144 * 1024;

template <int KMAX, int DMAX, bool ADAPT>
int launch_fast_t(const SelKArgs& a, int batch, hipStream_t s) {
    SelKArgs k = a;
    k.rehearse = fast_lds_bytes(a.rows_per_seq, KMAX, DMAX, true) <= kFastLdsLimit ? 1 : 0;
    const size_t lds = fast_lds_bytes(a.rows_per_seq, KMAX, DMAX, k.rehearse != 0);
    int st = set_lds(tree_fast_kernel<KMAX, DMAX, ADAPT>, lds);
    if (st != OT_OK) return st;
    hipLaunchKernelGGL((tree_fast_kernel<KMAX, DMAX, ADAPT>), dim3(batch), dim3(256), lds, s, k.row_topv, k.row_lse, k.k,
                       k.rows_per_seq, k);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}
template <int KMAX, bool ADAPT>
int launch_fast_k(const SelKArgs& a, int batch, hipStream_t s) {
    if (a.depth <= 8) return launch_fast_t<KMAX, 8, ADAPT>(a, batch, s);
    if (a.depth <= 10) return launch_fast_t<KMAX, 10, ADAPT>(a, batch, s);
    if (a.depth <= 12) return launch_fast_t<KMAX, 12, ADAPT>(a, batch, s);
    if (a.depth <= 16) return launch_fast_t<KMAX, 16, ADAPT>(a, batch, s);
    if (a.depth <= 20) return launch_fast_t<KMAX, 20, ADAPT>(a, batch, s);
    return launch_fast_t<KMAX, 32, ADAPT>(a, batch, s);
}
template <bool ADAPT>
int launch_fast(const SelKArgs& a, int batch, hipStream_t s) {
    if (a.k <= 4) return launch_fast_k<4, ADAPT>(a, batch, s);
    if (a.k <= 8) return launch_fast_k<8, ADAPT>(a, batch, s);
    if (a.k <= 10) return launch_fast_k<10, ADAPT>(a, batch, s);
    return launch_fast_k<16, ADAPT>(a, batch, s);
}
int fast_kmax(int k) { return k <= 4 ? 4 : (k <= 8 ? 8 : (k <= 10 ? 10 : 16)); }
int fast_dmax(int d) { return d <= 8 ? 8 : (d <= 10 ? 10 : (d <= 12 ? 12 : (d <= 16 ? 16 : (d <= 20 ? 20 : 32)))); }

}  // namespace

int launch_tree_oneshot(const SelectGeometry& g, const BuildWorkspace& ws, const ot_tree_out& out, hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.out = out;
    if (g.n <= 64 && fast_lds_bytes(g.rows_per_seq, fast_kmax(g.k), fast_dmax(g.depth), false) <= kFastLdsLimit)
        return launch_fast<false>(a, g.batch, s);
    const int NT = threads_for(g.n);
    return NT == 64 ? launch_oneshot_s<true>(a, g.batch, NT, s) : launch_oneshot_s<false>(a, g.batch, NT, s);
}

bool tree_adaptive_supported(const SelectGeometry& g) {
    return g.n <= 64 && fast_lds_bytes(g.rows_per_seq, fast_kmax(g.k), fast_dmax(g.depth), false) <= kFastLdsLimit;
}

int launch_tree_adaptive(const SelectGeometry& g, double delta, const BuildWorkspace& ws, const ot_tree_out& out,
                         int32_t* steps_used, double* e_sub, hipStream_t s) {
    if (!tree_adaptive_supported(g)) return OT_ERR_UNSUPPORTED;
    SelKArgs a = make_args(g, ws);
    a.out = out; a.delta = delta; a.steps_used = steps_used; a.e_sub = e_sub;
    return launch_fast<true>(a, g.batch, s);
}

int launch_tree_step(const SelectGeometry& g, int step, const BuildWorkspace& ws, int32_t* frontier_token,
                     int32_t* frontier_parent, int32_t* frontier_count, hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.step = step;
    a.frontier_token = frontier_token; a.frontier_parent = frontier_parent; a.frontier_count = frontier_count;
    const int NT = threads_for(g.n);
    return NT == 64 ? launch_step_s<true>(a, g.batch, NT, s) : launch_step_s<false>(a, g.batch, NT, s);
}

template <int DMAX, bool SINGLE>
int launch_esub_t(const SelKArgs& a, int batch, int NT, hipStream_t s) {
    const size_t lds = pool_lds_bytes(a.depth, NT, DMAX, 0);
    int st = set_lds(tree_esub_kernel<DMAX, SINGLE>, lds);
    if (st != OT_OK) return st;
    hipLaunchKernelGGL((tree_esub_kernel<DMAX, SINGLE>), dim3(batch), dim3(NT), lds, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

int launch_tree_begin(const SelectGeometry& g, const BuildWorkspace& ws, hipStream_t s) {
    hipLaunchKernelGGL(tree_begin_kernel, dim3((g.batch + 255) / 256), dim3(256), 0, s, ws.seq_E, ws.seq_steps,
                       ws.seq_active, g.batch);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

int launch_tree_esub(const SelectGeometry& g, int steps_done, double delta, const BuildWorkspace& ws, double* e_sub,
                     int32_t* go_on, hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.step = steps_done; a.delta = delta; a.e_sub = e_sub; a.go_on = go_on;
    const int NT = threads_for(g.n);
    if (NT == 64) {
        if (steps_done <= 8) return launch_esub_t<8, true>(a, g.batch, NT, s);
        if (steps_done <= 16) return launch_esub_t<16, true>(a, g.batch, NT, s);
        return launch_esub_t<32, true>(a, g.batch, NT, s);
    }
    if (steps_done <= 8) return launch_esub_t<8, false>(a, g.batch, NT, s);
    if (steps_done <= 16) return launch_esub_t<16, false>(a, g.batch, NT, s);
    return launch_esub_t<32, false>(a, g.batch, NT, s);
}

int launch_tree_front_mask(const SelectGeometry& g, int steps_done, const BuildWorkspace& ws, uint64_t* mask_out,
                           int mask_words, hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.step = steps_done; a.mask_out = (u64*)mask_out; a.mask_words = mask_words;
    hipLaunchKernelGGL(tree_front_mask_kernel, dim3(g.batch), dim3(256), 0, s, a);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

int launch_tree_finalize(const SelectGeometry& g, int steps_done, const BuildWorkspace& ws, const ot_tree_out& out,
                         hipStream_t s) {
    SelKArgs a = make_args(g, ws);
    a.out = out;
    a.step = steps_done;
    const int NT = threads_for(g.n);
    if (NT == 64) {
        if (steps_done <= 8) return launch_finalize_t<8, true>(a, g.batch, NT, s);
        if (steps_done <= 16) return launch_finalize_t<16, true>(a, g.batch, NT, s);
        return launch_finalize_t<32, true>(a, g.batch, NT, s);
    }
    if (steps_done <= 8) return launch_finalize_t<8, false>(a, g.batch, NT, s);
    if (steps_done <= 16) return launch_finalize_t<16, false>(a, g.batch, NT, s);
    return launch_finalize_t<32, false>(a, g.batch, NT, s);
}

}  // namespace ot
