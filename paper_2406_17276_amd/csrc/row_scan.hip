// Row scan: for every logits row of the draft model, one pass over the row yields
//   lse  = log sum_v exp(x_v)            (normaliser of p_d = softmax(row), Sec. 2 "Inference")
//   top-k tokens by logit, equal logits -> smaller token id   (children of a node, Sec. 3 after Eq. 2)
// This is the HBM-bound part of tree construction: every element is read exactly once,
// 16 bytes per lane per load, and held in registers for both the maximum and the exp-sum.
//
// One workgroup handles one "part" (<= 32768 elements) of one row.  Inside a workgroup:
//   1. every lane loads its 32 elements (all loads are issued before the first use),
//   2. every wavefront, on its own: lane maxima -> wave maximum m_w, then s_w = sum exp(x - m_w)
//      over its registers (no workgroup barrier before this, so wavefronts whose data arrived
//      early do their arithmetic while the others still wait for memory),
//   3. barrier; tau = the k-th largest of the group maxima (a group = a row of 16 lanes, 64 groups in a
//      1024-thread workgroup): each group holds an element >= its maximum, so at least k elements are >= tau,
//   4. sweep over the registers: elements >= tau go to an LDS candidate list (a 16-byte vector is
//      skipped when its own maximum is below tau),
//   5. the k best candidates are ranked by counting (value desc, token asc); the wave partials are
//      combined in fp64: M = max m_w, s = sum s_w exp(m_w - M), lse = M + log s,
//   6. part results are written; rows split over several parts are merged by merge_parts_kernel.
// If the candidate list overflows (massive ties), a slow exact path extracts the k best
// by k rounds of a workgroup-wide arg-max over the part, re-read from memory.
#include "common.hpp"
#include <type_traits>

namespace ot {
namespace {

constexpr int kCandCap = 2048;
constexpr float kLog2e = 1.4426950408889634f;
constexpr long long kScanMaxGrid = 16384;      // workgroups per launch; more items are walked with a grid stride

struct ScanKArgs {
    int vocab, k, parts, part_elems;
    int items;                        // rows x parts
    // P == 1: final row results; P > 1: per-part results
    double* row_lse; float* row_topv; int32_t* row_topi;
    float* part_m; double* part_s; float* part_topv; int32_t* part_topi;
    const int32_t* seq_active;        // SKIP kernels: rows of sequence b are left unread when seq_active[b] == 0
};

__device__ __forceinline__ unsigned int f32_key(float v) {
    unsigned int u = __float_as_uint(v);
    return (u >> 31) ? ~u : (u | 0x80000000u);
}

// What a work item needs to find its logits.  The kernels take these as leading scalar arguments, which the
// hardware hands over in registers at wavefront start (kernel-argument preload): the loads of a work item go out
// without waiting for a read of the argument block.
struct ScanHead {
    const void* logits;
    long long stride_seq, stride_depth, stride_row;
    int vocab;
    int part_geom;                    // parts | part_elems << 4
    int rows_per_seq;
    int grow;                         // nsteps | k << 8 | n << 16: step t covers F_t rows, F_0 = 1, F_{t+1} = min(n, k F_t)
};

// One work item = one row part (a whole row when the vocabulary fits one part).
template <int DT, int NT, int EPL, bool VECLOAD>
__device__ __forceinline__ void scan_item(const ScanHead& h, const ScanKArgs& a, const int wg) {
    constexpr int VEC = (DT == OT_BF16) ? 8 : 4;   // elements per 16-byte vector; EPL = elements per lane
    constexpr int VPL = EPL / VEC;      // 16-byte vectors per lane
    constexpr int NW = NT / 64;

    constexpr int G = NT / 16;          // groups for the threshold: the rows of 16 lanes (16, 32 or 64 of them)
    __shared__ float s_gmax[G];
    __shared__ float s_wm[16];
    __shared__ double s_ws[16];
    __shared__ float s_tau;
    __shared__ float s_cv[kCandCap];
    __shared__ int s_ci[kCandCap];
    __shared__ int s_rank[kCandCap];
    __shared__ int s_count;
    __shared__ unsigned long long s_best[16];

    const int tid = threadIdx.x;
    const int parts = h.part_geom & 15, part_elems = h.part_geom >> 4;
    const int rid = wg / parts;
    const int part = wg - rid * parts;
    const int b = rid / h.rows_per_seq;
    const int r = rid - b * h.rows_per_seq;
    // row r of a sequence is slot j of step t (Algorithm 1: the frontier grows k-fold per step up to n)
    const int nsteps = h.grow & 255, grow_k = (h.grow >> 8) & 255, grow_n = h.grow >> 16;
    int t = 0, start = 0, F = 1;
    while (t + 1 < nsteps && r >= start + F) {
        start += F;
        F = min(grow_n, grow_k * F);
        ++t;
    }
    const int j = r - start;
    const long long row_off = (long long)b * h.stride_seq + (long long)t * h.stride_depth + (long long)j * h.stride_row;
    const int e_begin = part * part_elems;
    const int e_end = min(h.vocab, e_begin + part_elems);

    if (tid == 0) s_count = 0;

    // ---- 1. load ----------------------------------------------------------
    // VECLOAD: the host guarantees 16-byte aligned rows and vocab % VEC == 0, so a vector is
    // either wholly inside the part or wholly outside.  A lane's address is (uniform start of the part) + (a 32-bit
    // byte offset); lanes past the end of the part re-read the part's first vector and are set to -inf afterwards,
    // which only the part's last vectors need (a uniform test).  Otherwise: guarded scalar loads.
    float x[EPL];
    const int len = e_end - e_begin;
    if (VECLOAD) {
        typedef typename std::conditional<DT == OT_BF16, u32x4, f32x4>::type vec_t;
        constexpr int ESIZE = DT == OT_BF16 ? 2 : 4;
        const char* part = (const char*)h.logits + (row_off + e_begin) * ESIZE;
        vec_t w[VPL];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {                   // all loads go out before the first use
            const int e = (i * NT + tid) * VEC;
            w[i] = __builtin_nontemporal_load((const vec_t*)(part + (e < len ? (unsigned int)e * ESIZE : 0u)));
        }
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            if ((i + 1) * NT * VEC > len) {
                asm volatile("");      // keeps this a branch: full vectors skip the selects
                const bool have = (i * NT + tid) * VEC < len;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (DT == OT_BF16) w[i][c] = have ? w[i][c] : 0xff80ff80u;     // a pair of -inf
                    else               w[i][c] = have ? w[i][c] : -INFINITY;
                }
            }
            if (DT == OT_BF16) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    x[i * 8 + 2 * c] = bf16_lo((uint32_t)w[i][c]);
                    x[i * 8 + 2 * c + 1] = bf16_hi((uint32_t)w[i][c]);
                }
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) x[i * 4 + c] = (float)w[i][c];
            }
        }
    } else if (DT == OT_BF16) {
        const unsigned short* row = (const unsigned short*)h.logits + row_off;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int e0 = e_begin + (i * NT + tid) * VEC;
#pragma unroll
            for (int c = 0; c < VEC; ++c)
                x[i * 8 + c] = (e0 + c < e_end) ? __uint_as_float((unsigned)row[e0 + c] << 16) : -INFINITY;
        }
    } else {
        const float* row = (const float*)h.logits + row_off;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int e0 = e_begin + (i * NT + tid) * VEC;
#pragma unroll
            for (int c = 0; c < VEC; ++c) x[i * 4 + c] = (e0 + c < e_end) ? row[e0 + c] : -INFINITY;
        }
    }

    // ---- 2. per-wavefront statistics -------------------------------------
    float vmax[VPL];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        float v = x[i * VEC];
#pragma unroll
        for (int c = 1; c < VEC; ++c) v = fmaxf(v, x[i * VEC + c]);
        vmax[i] = v;
    }
    float m = vmax[0];
#pragma unroll
    for (int i = 1; i < VPL; ++i) m = fmaxf(m, vmax[i]);
    const float rmax = row16_max(m);                  // max of this lane's row of 16 lanes
    const float m_w = fmaxf(fmaxf(rl_f(rmax, 0), rl_f(rmax, 16)), fmaxf(rl_f(rmax, 32), rl_f(rmax, 48)));
    // e^(x - m) = 2^(x log2e - mc) with mc = fl(m log2e): one fma per element.  mc is carried along as the
    // wave's reference exponent, so its rounding cancels when the partial sums are combined.
    const float mc_w = m_w * kLog2e;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (m_w > -INFINITY) {
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i & 3] += __builtin_amdgcn_exp2f(fmaf(x[i], kLog2e, -mc_w));
    }
    const double s_w = wave_sum_rows_d((acc[0] + acc[1]) + (acc[2] + acc[3]));
    const int lane = tid & 63, wave = tid >> 6;
    if (lane == 0) { s_wm[wave] = mc_w; s_ws[wave] = s_w; }     // (reference exponent in log2 units, sum)
    // group maxima: a group is a row of 16 lanes
    if ((lane & 15) == 0) s_gmax[tid >> 4] = rmax;
    __syncthreads();

    // ---- 3. tau: the kk-th largest of the G group maxima -------------------
    // Every group holds an element >= its maximum, so at least kk elements are >= tau; the more groups, the
    // tighter the threshold (k = 16 over 16 groups would take the smallest maximum and let several times k
    // elements through).  Wavefront w ranks maxima w, w + NW, ...: one ballot per maximum, all wavefronts at once.
    {
        const int kk = a.k < G ? a.k : G;
        const float mine = lane < G ? s_gmax[lane] : -INFINITY;
#pragma unroll
        for (int q = wave; q < G; q += NW) {
            const float v = s_gmax[q];
            const unsigned long long before = __ballot(lane < G && (mine > v || (mine == v && lane < q)));
            if (__popcll(before) == kk - 1 && lane == 0) s_tau = v;
        }
    }
    __syncthreads();
    const float tau = s_tau;

    // ---- 4. candidates -----------------------------------------------------
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        if (vmax[i] >= tau) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const float v = x[i * VEC + c];
                const int e = e_begin + (i * NT + tid) * VEC + c;
                if (v >= tau && e < e_end) {
                    const int p = atomicAdd(&s_count, 1);
                    if (p < kCandCap) { s_cv[p] = v; s_ci[p] = e; }
                }
            }
        }
    }
    __syncthreads();
    const int ncand = s_count;

    // where the k winners of this part go
    float* outv; int32_t* outi;
    if (a.parts == 1) {
        outv = a.row_topv + (size_t)rid * a.k;
        outi = a.row_topi + (size_t)rid * a.k;
    } else {
        outv = a.part_topv + (size_t)wg * a.k;
        outi = a.part_topi + (size_t)wg * a.k;
    }
    // ---- 5a. combine the wave partials in fp64 (last wavefront, 16 lanes) --
    if (wave == NW - 1 && lane < 16) {
        const bool have = lane < NW;
        const float mw = have ? s_wm[lane] : -INFINITY;
        float M = mw;
        M = fmaxf(M, __int_as_float(dpp_i<DPP_QUAD_XOR1>(__float_as_int(M), __float_as_int(M))));
        M = fmaxf(M, __int_as_float(dpp_i<DPP_QUAD_XOR2>(__float_as_int(M), __float_as_int(M))));
        M = fmaxf(M, __int_as_float(dpp_i<DPP_ROW_HALF_MIRROR>(__float_as_int(M), __float_as_int(M))));
        M = fmaxf(M, __int_as_float(dpp_i<DPP_ROW_MIRROR>(__float_as_int(M), __float_as_int(M))));
        double part_sum = (have && mw > -INFINITY) ? s_ws[lane] * (double)__builtin_amdgcn_exp2f(mw - M) : 0.0;
        part_sum += dpp_d<DPP_QUAD_XOR1>(part_sum);
        part_sum += dpp_d<DPP_QUAD_XOR2>(part_sum);
        part_sum += dpp_d<DPP_ROW_HALF_MIRROR>(part_sum);
        part_sum += dpp_d<DPP_ROW_MIRROR>(part_sum);
        if (lane == 0) {
            if (a.parts == 1) {
                // the terms are 2^(x c - M) with c = the fp32 constant, i.e. e^((x - M / c) c / log2e): dividing
                // M by the same c puts the reference back into natural-log units without a bias in the constant
                a.row_lse[rid] = (double)M / (double)kLog2e + log(part_sum);
            } else {
                a.part_m[wg] = M;
                a.part_s[wg] = part_sum;
            }
        }
    }

    // ---- 5b. rank the candidates -------------------------------------------
    if (ncand <= kCandCap) {
        constexpr int PR = NT >= 1024 ? 32 : 16;          // PR x PR pairs fit the workgroup
        if (ncand <= PR && NT >= PR * PR) {
            // one (candidate i, rival j) pair per thread: rank of i = rivals that precede it, counted with a ballot
            const int i = tid / PR, j = tid % PR;
            if (tid < PR * PR) {
                const float v = s_cv[i < ncand ? i : 0], u = s_cv[j < ncand ? j : 0];
                const int id = s_ci[i < ncand ? i : 0], ui = s_ci[j < ncand ? j : 0];
                const unsigned long long bal = __ballot(j < ncand && (u > v || (u == v && ui < id)));
                // a wavefront holds 64 / PR candidates, PR consecutive lanes each
                const int rank = __popcll(PR == 32 ? ((lane & 32) ? (bal >> 32) : (bal & 0xffffffffull))
                                                   : ((bal >> (lane & 48)) & 0xffffull));
                if (j == 0 && i < ncand && rank < a.k) { outv[rank] = v; outi[rank] = id; }
            }
            return;
        }
        if (ncand <= 64 && NT >= 1024) {
            // 64 x 64 pairs: thread = (candidate i, 4 rivals); the 16 threads of a candidate share a row of lanes
            const int i = tid >> 4, j0 = (tid & 15) * 4;
            const float v = s_cv[i < ncand ? i : 0];
            const int id = s_ci[i < ncand ? i : 0];
            int cnt = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int jj = j0 + c;
                const float u = s_cv[jj < ncand ? jj : 0];
                const int ui = s_ci[jj < ncand ? jj : 0];
                cnt += (jj < ncand && (u > v || (u == v && ui < id))) ? 1 : 0;
            }
            cnt += dpp_i<DPP_QUAD_XOR1>(0, cnt);
            cnt += dpp_i<DPP_QUAD_XOR2>(0, cnt);
            cnt += dpp_i<DPP_ROW_HALF_MIRROR>(0, cnt);
            cnt += dpp_i<DPP_ROW_MIRROR>(0, cnt);
            if ((tid & 15) == 0 && i < ncand && cnt < a.k) { outv[cnt] = v; outi[cnt] = id; }
            return;
        }
        if (ncand <= 64) {
            if (wave == 0) {          // candidate i sits in lane i; the others are broadcast by v_readlane
                const float v = lane < ncand ? s_cv[lane] : -INFINITY;
                const int id = lane < ncand ? s_ci[lane] : 0x7fffffff;
                int rank = 0;
                for (int jj = 0; jj < ncand; ++jj) {
                    const float u = rl_f(v, jj);
                    const int ui = rl(id, jj);
                    rank += (u > v || (u == v && ui < id)) ? 1 : 0;
                }
                if (lane < ncand && rank < a.k) { outv[rank] = v; outi[rank] = id; }
            }
            return;
        }
        for (int i = tid; i < kCandCap; i += NT) s_rank[i] = 0;
        __syncthreads();
        int cp = 64;
        while (cp < ncand) cp <<= 1;
        const int q_cnt = (NT / cp) > 0 ? (NT / cp) : 1;   // slices of the inner loop per candidate
        if (cp <= NT) {
            const int i = tid & (cp - 1);
            const int q = tid / cp;
            if (i < ncand) {
                const float v = s_cv[i];
                const int id = s_ci[i];
                int rank = 0;
                for (int jj = q; jj < ncand; jj += q_cnt) {
                    const float u = s_cv[jj];
                    const int ui = s_ci[jj];
                    rank += (u > v || (u == v && ui < id)) ? 1 : 0;
                }
                if (q_cnt > 1) atomicAdd(&s_rank[i], rank); else s_rank[i] = rank;
            }
        } else {
            for (int i = tid; i < ncand; i += NT) {
                const float v = s_cv[i];
                const int id = s_ci[i];
                int rank = 0;
                for (int jj = 0; jj < ncand; ++jj) {
                    const float u = s_cv[jj];
                    const int ui = s_ci[jj];
                    rank += (u > v || (u == v && ui < id)) ? 1 : 0;
                }
                s_rank[i] = rank;
            }
        }
        __syncthreads();
        for (int i = tid; i < ncand; i += NT) {
            const int rank = s_rank[i];
            if (rank < a.k) { outv[rank] = s_cv[i]; outi[rank] = s_ci[i]; }
        }
        return;
    }

    // ---- slow exact path: k rounds of arg-max, re-reading the part from memory ----
    float prev_v = INFINITY;
    int prev_i = -1;
    for (int round = 0; round < a.k; ++round) {
        unsigned long long best = 0ull;
        for (int e = e_begin + tid; e < e_end; e += NT) {
            float v;
            if (DT == OT_BF16) v = __uint_as_float((unsigned)((const unsigned short*)h.logits + row_off)[e] << 16);
            else v = ((const float*)h.logits + row_off)[e];
            const bool after = (v < prev_v) || (v == prev_v && e > prev_i);
            if (after) {
                const unsigned long long key =
                    ((unsigned long long)f32_key(v) << 32) | (unsigned long long)(0xffffffffu - (unsigned)e);
                best = key > best ? key : best;
            }
        }
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long other = __shfl_xor(best, o);
            best = other > best ? other : best;
        }
        __syncthreads();
        if ((tid & 63) == 0) s_best[tid >> 6] = best;
        __syncthreads();
        best = s_best[0];
        for (int w = 1; w < NW; ++w) best = s_best[w] > best ? s_best[w] : best;
        if (best == 0ull) break;      // fewer than k valid elements in this part
        const unsigned int fk = (unsigned int)(best >> 32);
        const unsigned int fu = (fk >> 31) ? (fk & 0x7fffffffu) : ~fk;
        prev_v = __uint_as_float(fu);
        prev_i = (int)(0xffffffffu - (unsigned)(best & 0xffffffffu));
        if (tid == 0) { outv[round] = prev_v; outi[round] = prev_i; }
    }
}

// Launches of up to kScanMaxGrid items have one workgroup per item; larger ones (long-vocabulary, large-batch
// shapes with 10^5..10^6 items) are walked with a grid stride, because starting a workgroup costs about as
// much as a small item's share of the memory traffic.
// SKIP: the scan of one drafting step in the loop of Algorithm 1 -- a sequence that the stopping rule has frozen
// drafts no further, and its rows are not read (the flag is the step kernel's own, on the device).
__device__ __forceinline__ bool scan_item_frozen(const ScanKArgs& a, int part_geom, int rows_per_seq, int wg) {
    const int rid = wg / (part_geom & 15);
    return a.seq_active[rid / rows_per_seq] == 0;
}
template <int DT, int NT, int EPL, bool VECLOAD, bool SKIP>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu((NT == 1024 && VECLOAD) ? 8 : 4, 8))) void row_scan_kernel(
    const void* logits, const long long stride_seq, const long long stride_depth, const long long stride_row,
    const int vocab, const int part_geom, const int rows_per_seq, const int grow, const ScanKArgs a) {
    if (SKIP && scan_item_frozen(a, part_geom, rows_per_seq, blockIdx.x)) return;
    const ScanHead h{logits, stride_seq, stride_depth, stride_row, vocab, part_geom, rows_per_seq, grow};
    scan_item<DT, NT, EPL, VECLOAD>(h, a, blockIdx.x);
}
template <int DT, int NT, int EPL, bool VECLOAD, bool SKIP>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu((NT == 1024 && VECLOAD) ? 8 : 4, 8))) void row_scan_strided_kernel(
    const void* logits, const long long stride_seq, const long long stride_depth, const long long stride_row,
    const int vocab, const int part_geom, const int rows_per_seq, const int grow, const ScanKArgs a) {
    const ScanHead h{logits, stride_seq, stride_depth, stride_row, vocab, part_geom, rows_per_seq, grow};
    for (int wg = blockIdx.x; wg < a.items; wg += gridDim.x) {
        if (SKIP && scan_item_frozen(a, part_geom, rows_per_seq, wg)) continue;      // (the whole workgroup skips)
        scan_item<DT, NT, EPL, VECLOAD>(h, a, wg);
        if (wg + (int)gridDim.x < a.items) __syncthreads();      // the next item reuses the shared arrays
    }
}

// Rows that span several parts: combine the per-part (max, sum) pairs and merge the per-part top-k lists.
// One wavefront per row: the parts' statistics sit in the first lanes, the parts * k <= 128 candidates go through
// LDS and every lane ranks its (at most two) candidates by counting those that precede them (value desc, token
// asc: tokens of different parts differ, so the order is total); ranks below k are the row's list.
__global__ __launch_bounds__(256) void merge_parts_kernel(int rows, int parts, int k, const float* part_m,
                                                          const double* part_s, const float* part_topv,
                                                          const int32_t* part_topi, double* row_lse, float* row_topv,
                                                          int32_t* row_topi) {
    __shared__ float s_v[4][128];
    __shared__ int s_i[4][128];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int rid = blockIdx.x * 4 + w;
    const bool live = rid < rows;
    const size_t base = (size_t)(live ? rid : 0) * parts;
    const int total = parts * k;
    // part_m is the part's reference exponent in log2 units (fp32 max times the fp32 log2e of the scan kernel)
    const float pm = lane < parts ? part_m[base + lane] : -INFINITY;
    const float M = wave_max(pm);
    const double s = wave_sum(lane < parts ? part_s[base + lane] * exp2((double)pm - (double)M) : 0.0);
    if (live && lane == 0) row_lse[rid] = (double)M / (double)kLog2e + log(s);
    for (int c = lane; c < total; c += 64) {               // the row's lists are contiguous: part p, rank r at p k + r
        s_v[w][c] = part_topv[base * k + c];
        s_i[w][c] = part_topi[base * k + c];
    }
    __syncthreads();
    float v[2]; int id[2], rank[2] = {0, 0};
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int c = lane + 64 * q;
        v[q] = c < total ? s_v[w][c] : -INFINITY;
        id[q] = c < total ? s_i[w][c] : 0x7fffffff;
    }
    for (int j = 0; j < total; ++j) {
        const float u = s_v[w][j];
        const int ui = s_i[w][j];
#pragma unroll
        for (int q = 0; q < 2; ++q) rank[q] += (u > v[q] || (u == v[q] && ui < id[q])) ? 1 : 0;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
        if (live && lane + 64 * q < total && rank[q] < k) {
            row_topv[(size_t)rid * k + rank[q]] = v[q];
            row_topi[(size_t)rid * k + rank[q]] = id[q];
        }
}

}  // namespace

int launch_row_scan(const ScanGeometry& g, const void* logits, const BuildWorkspace& ws, hipStream_t s, hipEvent_t ev0,
                    hipEvent_t ev1, bool skip_frozen) {
    const int parts = scan_parts(g.vocab);
    if (parts > 8) return OT_ERR_UNSUPPORTED;
    const int esize = g.dtype == OT_BF16 ? 2 : 4;
    const int vec = 16 / esize;
    ScanKArgs a;
    a.vocab = g.vocab; a.k = g.k; a.parts = parts;
    const int per = (g.vocab + parts - 1) / parts;
    a.part_elems = (per + vec - 1) / vec * vec;
    if (g.nsteps < 1 || g.nsteps > 255 || g.grow_k < 1 || g.grow_k > 255 || g.grow_n < 1 || g.grow_n > 32767)
        return OT_ERR_INVALID_ARG;
    const int part_geom = parts | (a.part_elems << 4);
    const int grow = g.nsteps | (g.grow_k << 8) | (g.grow_n << 16);
    a.row_lse = ws.row_lse; a.row_topv = ws.row_topv; a.row_topi = ws.row_topi;
    a.part_m = ws.part_m; a.part_s = ws.part_s; a.part_topv = ws.part_topv; a.part_topi = ws.part_topi;
    a.seq_active = skip_frozen ? ws.seq_active : nullptr;

    const bool aligned = ((uintptr_t)logits % 16 == 0) && (g.stride_seq % vec == 0) && (g.stride_depth % vec == 0) &&
                         (g.stride_row % vec == 0) && (g.vocab % vec == 0);
    const bool small = a.part_elems <= 256 * 32;
    const long long rows = (long long)g.batch * g.rows_per_seq;
    const long long grid = rows * parts;
    if (grid <= 0 || grid > 0x7fffffffLL) return OT_ERR_UNSUPPORTED;
    a.items = (int)grid;
    const dim3 gd((unsigned)(grid <= kScanMaxGrid ? grid : kScanMaxGrid));

#define OT_SCAN_ARGS logits, g.stride_seq, g.stride_depth, g.stride_row, g.vocab, part_geom, g.rows_per_seq, grow, a
#define OT_SCAN_LAUNCH2(DT, NT, VL, SK)                                                                  \
    do {                                                                                                 \
        if (grid > kScanMaxGrid) {                                                                       \
            if (ev0 || ev1) hipExtLaunchKernelGGL((row_scan_strided_kernel<DT, NT, 32, VL, SK>), gd, dim3(NT), 0, s, ev0, ev1, 0, OT_SCAN_ARGS); \
            else hipLaunchKernelGGL((row_scan_strided_kernel<DT, NT, 32, VL, SK>), gd, dim3(NT), 0, s, OT_SCAN_ARGS);   \
        } else if (ev0 || ev1) hipExtLaunchKernelGGL((row_scan_kernel<DT, NT, 32, VL, SK>), gd, dim3(NT), 0, s, ev0, ev1, 0, OT_SCAN_ARGS); \
        else hipLaunchKernelGGL((row_scan_kernel<DT, NT, 32, VL, SK>), gd, dim3(NT), 0, s, OT_SCAN_ARGS);               \
    } while (0)
#define OT_SCAN_LAUNCH(DT, NT, VL) do { if (skip_frozen) OT_SCAN_LAUNCH2(DT, NT, VL, true); else OT_SCAN_LAUNCH2(DT, NT, VL, false); } while (0)
    if (g.dtype == OT_BF16) {
        if (small) { if (aligned) OT_SCAN_LAUNCH(OT_BF16, 256, true); else OT_SCAN_LAUNCH(OT_BF16, 256, false); }
        else       { if (aligned) OT_SCAN_LAUNCH(OT_BF16, 1024, true); else OT_SCAN_LAUNCH(OT_BF16, 1024, false); }
    } else {
        if (small) { if (aligned) OT_SCAN_LAUNCH(OT_F32, 256, true); else OT_SCAN_LAUNCH(OT_F32, 256, false); }
        else       { if (aligned) OT_SCAN_LAUNCH(OT_F32, 1024, true); else OT_SCAN_LAUNCH(OT_F32, 1024, false); }
    }
#undef OT_SCAN_LAUNCH2
#undef OT_SCAN_LAUNCH
#undef OT_SCAN_ARGS
    OT_HIP_CHECK(hipGetLastError());
    if (parts > 1) {
        hipLaunchKernelGGL(merge_parts_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s,
                           (int)rows, parts, g.k, ws.part_m, ws.part_s, ws.part_topv, ws.part_topi, ws.row_lse,
                           ws.row_topv, ws.row_topi);
        OT_HIP_CHECK(hipGetLastError());
    }
    return OT_OK;
}

}  // namespace ot
