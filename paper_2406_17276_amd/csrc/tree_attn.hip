// Tree-masked attention (Algorithm 2: the target model's forward over the drafted nodes with the tree
// attention mask; with n_keys > n also the draft model's attention of a drafting step, Sec. 4).
// For query row i of sequence b and query head h:
//   O[i] = sum_j softmax_j(scale q_i.k_j) v_j,  j over the cached prefix and the tree rows
//   whose bit is set in mask[b][i] (the node itself and its ancestors).
//
// The keys of one (sequence, KV head) are cut into 64-key tiles: ceil(L_b/64) prefix tiles,
// then ceil(n_keys/64) tree tiles.  Contiguous tile ranges ("splits") go to different workgroups so
// that a single small sequence still fills the chip; every split leaves an un-normalised
// partial (running max m, sum l, O).  The bf16 kernel merges the partials itself (the last workgroup
// of a row block to finish does it), the f32 kernel leaves them to attn_combine_kernel.
//
// bf16 path (attn_mfma_kernel): one workgroup = 64 or 128 packed query rows of one KV head (GQA: the
// g = q_heads/kv_heads query heads that share the KV head are stacked, row = head*n + node), four
// wavefronts.  Each wavefront
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q held in registers;
//                 the accumulator leaves every lane with 16 scores of ONE query, so the
//                 online-softmax statistics and the rescale factor are per-lane scalars;
//   O^T += V^T P^T  same instruction, B = P straight from the S^T accumulators (the key order
//                 inside a 16-key slab is whatever the accumulator layout gives; V is read in
//                 the same order), A = V gathered from LDS.
// K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4: 16 bytes per lane, no
// register staging), one or two tiles ahead of the computation, into a ring of two or three buffers; a tree
// tile's mask words (one 64-bit word per query row) travel the same way, just ahead of the tile.  A
// wavefront's 64 lanes land on 1 KB of consecutive LDS, so rows are unpadded and bank conflicts are
// avoided by an XOR swizzle instead: lane -> global chunk is chosen such that 16-byte chunk c of key
// row r sits at chunk position c ^ (r mod 16) (K), and 32-byte segment g of row r at g ^ v_swizzle(r) (V; see the kernel).
// Tiles that reach past the end of the keys re-read the last valid row for the missing rows (their scores
// are masked).  V is the transposed operand (a lane needs 8 keys of ONE column): it is read with the gfx950
// LDS transpose load ds_read_b64_tr_b16, which lets 16 lanes read four 32-byte row segments and hands
// lane i the i-th column of that 4x16 block -- two such loads per MFMA operand.
// The ancestor mask is applied bit by bit on tree tiles only (any number of tree keys: a tile needs one word per
// row); prefix tiles only mask the tail.  The kernel's first memory requests decide its length at the small
// shapes, so the prologue is kept short: divisions are multiplications by constants prepared on the host, the
// prefix length is fetched first, Q is requested before and the first tiles right after it is known.
//
// f32 path (attn_f32_kernel): plain fp32 FMA arithmetic, 16 query rows x 32-key tiles.
#include <math.h>

#include <mutex>
#include <type_traits>

#include "common.hpp"

namespace ot {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kMaxSplits = 32;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct AttnKArgs {
    const void *Q, *Kp, *Vp, *Kt, *Vt;
    const int32_t* prefix_len;
    const uint64_t* mask;
    void* O;
    unsigned int* counters;   // one ticket counter per (sequence, KV head, row block), zero between launches
    float* part_o;      // per-split partial O   (layout: see the kernel that writes it)
    float* part_ml;     // per-split (m, l)
    int batch, q_heads, kv_heads, g, n, nk, D, max_prefix, splits, W, dtype, row_blocks;   // n query rows, nk tree keys
    int splits_share_xcd;   // workgroup numbering of the bf16 kernel, see there
    unsigned int inv_splits, inv_kv_heads, inv_n;   // division by multiplication (fast_div): ceil(2^32 / d), unused for d = 1
    float scale_log2;   // softmax scale * log2(e)
    const float *k_scale, *v_scale;   // 8-bit K/V cache: one factor per (sequence, KV head) each; null otherwise
    long long qs[3], kps[3], vps[3], kts[3], vts[3], os[3];
};

// max over lanes l and l ^ 32 (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float xhalf_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ int clamp_len(int L, int maxp) { return L < 0 ? 0 : (L > maxp ? maxp : L); }

// A prefix length outside [0, max_prefix] is clamped and reported in the workspace's status word.
__device__ __forceinline__ void report_clamp(unsigned int* sync_words, int raw, int maxp) {
    if (raw < 0 || raw > maxp)
        __hip_atomic_fetch_or(sync_words + OT_ATTN_STATUS_OFFSET / 4, OT_ATTN_STATUS_PREFIX_CLAMPED, __ATOMIC_RELAXED,
                              __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until all but the N youngest memory requests of this lane have landed.  The Q fragments were requested
// with assembly the compiler does not track; they are in/out operands here, which places whatever reads them
// after this wait.  Executed once, ahead of the tile loop (straight-line code: the operands stay where they are).
template <int N, int SLABS>
__device__ __forceinline__ void wait_q(u32x4 (&q)[SLABS]) {
    static_assert(SLABS == 4 || SLABS == 8, "head_dim 64 or 128");
    if constexpr (SLABS == 8)
        asm volatile("s_waitcnt vmcnt(%8)"
                     : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]), "+v"(q[4]), "+v"(q[5]), "+v"(q[6]), "+v"(q[7])
                     : "n"(N) : "memory");
    else
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]) : "n"(N) : "memory");
}

// x / d for x d < 2^32 as one multiplication by M = ceil(2^32 / d), prepared on the host (an integer division
// costs some forty instructions here, and the kernel's first memory requests wait for several of them).
__device__ __forceinline__ int fast_div(int x, int d, unsigned int M) {
    return d == 1 ? x : (int)__umulhi((unsigned int)x, M);
}

// Tile range of split s out of S over T tiles (T s < 2^32 / S).
__device__ __forceinline__ void split_range(int T, int S, unsigned int inv_S, int s, int& t0, int& t1) {
    t0 = fast_div(T * s, S, inv_S);
    t1 = fast_div(T * (s + 1), S, inv_S);
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel
// ---------------------------------------------------------------------------
// WIDE = false: 64 packed rows per workgroup, wavefront = (query block of 32 rows) x (half of each
//                64-key tile); the two halves are merged through LDS at the end.  For few rows.
//                Three tile buffers: two tiles are in flight while a third is being computed.
// WIDE (VAR 1, 2): 128 or 256 packed rows per workgroup (four or eight wavefronts), wavefront = 32 rows x the whole tile; staging one
//                tile in LDS is shared by twice as many MFMAs and nothing is merged at the end.
//                Two tile buffers, so that two workgroups share a compute unit.
// Workgroups are numbered so that those which stream the same K/V (the row blocks of one
// (sequence, KV head, split)) sit on the same XCD, next to each other in its dispatch order, and
// share that XCD's L2: hardware hands workgroup L to XCD L % 8.  When the (sequence, KV head) pairs divide evenly
// over the eight XCDs, the key splits of a pair share an XCD as well: they read the same Q rows, which then come
// from memory once per pair instead of once per split.
//
// With more than one split, every workgroup leaves its partial (O, m, l) in the workspace in the
// accumulator's own register order (coalesced 16-byte stores), then takes a ticket from the counter
// of its (sequence, KV head, row block); the workgroup that draws the last ticket merges all the
// partials of those rows and writes O.  Nobody waits for anybody: a workgroup that is not last simply
// ends.  The counter is reset by the merging workgroup, so it is zero again when the kernel ends.
#ifndef OT_ATTN_NBUF_NARROW
#define OT_ATTN_NBUF_NARROW 3
#endif
// Partial results of the key splits travel as bf16 (0) or as fp32 (define to 0): bf16 halves the exchange and lets the
// merging workgroup hold all of a row block's partials in registers at once, one trip to memory instead of two; the
// extra rounding is of the size of the output's own (the output is bf16).
#ifndef OT_ATTN_PART_BF16
#define OT_ATTN_PART_BF16 1
#endif
// KV8: K and V arrive as FP8 E4M3 bytes with a scale factor per (sequence, KV head) each.  A tile is copied into LDS
// as it is (half the bytes), then every thread widens its sixteen-byte pieces to bf16 in place -- every E4M3 value
// is a bf16 value -- into the layout the operand reads expect (two more barriers per tile); the K factor joins the
// softmax scale, the V factor the final normalisation.  Everything else is the bf16 kernel.
//
// BAL (wide variants, batches of 2 to 64 sequences that fill the chip, each (sequence, KV head) in one piece): the
// sequences of a batch differ in length, workgroups are handed out in the order of their number, and a launch lasts
// as long as the compute unit that finishes last.  Every workgroup therefore reads all prefix lengths first (lane j
// = sequence j), ranks the sequences by length and takes the job that its number stands for in the order "longest
// first" -- the order in which handing jobs to whichever unit is free balances best.
template <int D, int VAR, bool KV8, bool BAL>
__global__ __launch_bounds__(VAR == 2 ? 512 : 256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_mfma_kernel(
    // what the first loads need, as leading scalar arguments: the hardware hands these over in registers at
    // wavefront start (kernel-argument preload); they repeat fields of `a`
    const int32_t* a_prefix_len, const uint64_t* a_mask, const void* a_Q, const int a_splits, const unsigned a_inv_splits,
    const int a_kv_heads, const unsigned a_inv_kv_heads, const int a_n, const unsigned a_inv_n, const AttnKArgs a) {
    const int a_g = a.g, a_max_prefix = a.max_prefix, a_nk = a.nk, a_W = a.W, a_row_blocks = a.row_blocks;
    constexpr bool WIDE = VAR >= 1;
    constexpr int NWAVES = VAR == 2 ? 8 : 4;
    constexpr int NT = 64 * NWAVES;        // threads
    constexpr int TK = 64;                 // keys per tile
    constexpr int CPR = D / 8;             // 16-byte chunks per row
    constexpr int SPR = D / 16;            // 32-byte segments per row
    // Where V's 32-byte segment g of key row r sits inside the row: at g ^ v_swizzle(r).  A transposed operand read
    // touches, per 32 lanes, four consecutive rows (r mod 4 = 0..3) and the two halves of a 32-column block (segments
    // 2d and 2d + 1); LDS serves 256 bytes = eight segments per cycle, so these eight must fall into eight different
    // 32-byte slots of a 256-byte window: the row's low bits go into the bits above the half bit (a plain g ^ (r mod 8)
    // put two of them into every slot it used: every such read took twice its time).
    auto v_swizzle = [](int r) { return D == 128 ? (r & 3) << 1 : ((r >> 1) & 1) << 1; };
    constexpr int SLABS = D / 16;          // 16-wide d slabs of the QK^T contraction
    constexpr int DB = D / 32;             // 32-wide d blocks of O^T
    constexpr int ESZ = KV8 ? 1 : 2;       // bytes per stored K/V element
    constexpr int CPRG = D * ESZ / 16;     // 16-byte chunks per row in global memory
    constexpr int CH = TK * CPRG / NT;     // 16-byte chunks per thread per tile (K or V)
    static_assert(CH >= 1, "a tile has at least one chunk per thread");
    constexpr int LPT = 2 * CH;            // asynchronous loads per thread per tile
    constexpr int NKB = WIDE ? 2 : 1;      // 32-key blocks per wavefront per tile
    constexpr int ROWS = VAR == 2 ? 256 : (WIDE ? 128 : 64);   // packed query rows per workgroup
    constexpr int NQB = ROWS / 32;         // query blocks per workgroup
    constexpr int NBUF = VAR == 2 ? 4 : (WIDE ? 2 : OT_ATTN_NBUF_NARROW);
    constexpr int PD = NBUF - 1;           // tiles requested ahead of the one being computed
    static_assert(PD >= 1 && PD <= 3 && PD * LPT < 64, "prefetch depth fits the vmcnt counter");

    constexpr int BUF = TK * D;            // dwords of one staged tile: K [64][D] bf16, then V [64][D] bf16
    extern __shared__ __attribute__((aligned(16))) unsigned int s_buf[];   // [NBUF][BUF]
    __shared__ int s_last;
    constexpr int MST = DB * 16 + 4;       // floats per lane in the half-merge scratch (a multiple of four)
    static_assert(sizeof(unsigned int) * NBUF * BUF >= 2 * 64 * MST * 4, "merge scratch fits");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qb = WIDE ? wave : (wave & 1), kh = WIDE ? 0 : (wave >> 1);
    const int l32 = lane & 31, h = lane >> 5;
    // workgroup numbering: see above
    // grid (8 x row blocks, units / 8): hardware hands workgroups out with x running fastest
    const int xcd = blockIdx.x & 7, rb = blockIdx.x >> 3;
    int bz, split;
    int L_bal = 0;
    if constexpr (BAL) {
        static_assert(VAR >= 1, "wide variants only");
        const int B = a.batch;                                   // 2..64, one key range per (sequence, KV head)
        const int Lj = lane < B ? a_prefix_len[lane] : 0;
        const int Tj = lane < B ? clamp_len(Lj, a_max_prefix) : -1;
        int rank = 0;                                            // sequences ahead of sequence j: longer ones, and equally long ones before it
        for (int i = 0; i < B; ++i) {
            const int Ti = __builtin_amdgcn_readlane(Tj, i);
            rank += (Ti > Tj || (Ti == Tj && i < lane)) ? 1 : 0;
        }
        const int job = blockIdx.y * 8 + xcd;                    // position in the order longest first
        const int q = fast_div(job, a_kv_heads, a_inv_kv_heads);
        if (q >= B) return;
        const int b_sel = (int)__builtin_ctzll(__ballot(rank == q && lane < B));
        L_bal = __builtin_amdgcn_readlane(Lj, b_sel);
        bz = b_sel * a_kv_heads + (job - q * a_kv_heads);
        split = 0;
    } else if (a.splits_share_xcd) {
        // (sequence, KV head) pairs dealt round over the XCDs, all splits of a pair on the same one
        const int round = fast_div(blockIdx.y, a_splits, a_inv_splits);
        split = blockIdx.y - round * a_splits;
        bz = round * 8 + xcd;
        if (bz >= a.batch * a_kv_heads) return;
    } else {
        const int unit = blockIdx.y * 8 + xcd;
        if (unit >= a.batch * a_kv_heads * a_splits) return;
        bz = fast_div(unit, a_splits, a_inv_splits);
        split = unit - bz * a_splits;
    }
    const int b = fast_div(bz, a_kv_heads, a_inv_kv_heads), hk = bz - b * a_kv_heads;
    const int n = a_n;
    // the prefix length decides which tiles this workgroup streams: fetched first (a scalar load, ahead of the
    // hand-issued loads below), used only when the tile requests are built
    const int L_raw = BAL ? L_bal : a_prefix_len[b];

    // this lane's query row; lanes past the last row work on a copy of it and store nothing
    const int rho = rb * ROWS + qb * 32 + l32;         // packed row inside the KV head
    const bool row_ok = rho < a_g * n;
    const int rho_c = row_ok ? rho : a_g * n - 1;
    const int head = fast_div(rho_c, n, a_inv_n);
    const int hq = hk * a_g + head;
    const int node = rho_c - head * n;

    // Q fragments (B operand of S^T = K Q^T; lane holds Q[row][16 s + 8 h .. +7]) are requested first, as
    // assembly like the tile requests below: the compiler does not know that they are in flight, so nothing
    // waits for them until the first tile does (s_waitcnt in tile_step; loads complete in order, Q is the
    // oldest).  The registers are handed to that wait as in/out operands, which keeps every use behind it.
    u32x4 qw[SLABS];
    {
        const unsigned short* qrow = (const unsigned short*)a_Q + (long long)b * a.qs[0] + (long long)hq * a.qs[1] +
                                     (long long)node * a.qs[2] + 8 * h;
#pragma unroll
        for (int s = 0; s < SLABS; ++s)
            asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=&v"(qw[s]) : "v"(qrow), "n"(32 * s) : "memory");
    }
    // this lane's ancestor mask row: one 64-bit word per 64-key tree tile, requested with the tile and, like it,
    // delivered straight into LDS (s_mw: per buffer and wavefront the low words of the 64 lanes, then the high words)
    const uint64_t* const mask_row = a_mask + ((long long)b * n + node) * a_W;
    unsigned int* const s_mw = s_buf + NBUF * BUF;                      // [NBUF][waves][2][64]

    const unsigned char* kp = (const unsigned char*)a.Kp + ((long long)b * a.kps[0] + (long long)hk * a.kps[1]) * ESZ;
    const unsigned char* vp = (const unsigned char*)a.Vp + ((long long)b * a.vps[0] + (long long)hk * a.vps[1]) * ESZ;
    const unsigned char* kt = (const unsigned char*)a.Kt + ((long long)b * a.kts[0] + (long long)hk * a.kts[1]) * ESZ;
    const unsigned char* vt = (const unsigned char*)a.Vt + ((long long)b * a.vts[0] + (long long)hk * a.vts[1]) * ESZ;

    // transpose-load addressing: key row and first column this lane points at inside a 4-key x 32-column block
    const int tr_j = (lane & 15) >> 2, tr_q = 4 * (lane & 3);
    // swizzle terms of this lane's operand reads: K chunk (2s + h) of row l32 -> position (2s) ^ kx;
    // V segment (2d + g1) of row 4h + tr_j (mod 4) -> position (2d) ^ vx
    const int kx = h ^ (l32 & (CPR - 1));
    const int vx = ((lane >> 4) & 1) ^ v_swizzle(4 * h + tr_j);
    // scores are kept raw; p = 2^(c s - c m).  An 8-bit cache's K factor scales every score: it joins c.
    const float c = KV8 ? a.scale_log2 * a.k_scale[bz] : a.scale_log2;
    const float v_factor = KV8 ? a.v_scale[bz] : 1.f;
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 oacc[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[d][v] = 0.f;

    // LDS slot sigma = cc * NT + tid (16 bytes each) holds key row sigma / CPR, chunk position sigma % CPR;
    // the chunk stored there is the one the swizzle maps to that position.  KSTEP rows separate cc and cc+1,
    // a multiple of 16, so the swizzle term is the same for every cc.
    // (KV8: the copy is not swizzled -- slot sigma holds chunk sigma % CPRG of row sigma / CPRG -- the widening is.)
    constexpr int KSTEP = NT / CPRG;
    const int kkey0 = tid / CPRG, pc = tid % CPRG;
    const int kcol = KV8 ? pc * 16 : (pc ^ (kkey0 & (CPR - 1))) * 16;                        // byte column; K: chunk c = pc ^ (r % 16)
    const int vcol = KV8 ? pc * 16 : (2 * ((pc >> 1) ^ v_swizzle(kkey0)) + (pc & 1)) * 16;  // V: segment g = (pc/2) ^ v_swizzle(r)
    const int wave_u = wave;
    // Request tile t: global memory -> LDS buffer `buf`, 16 bytes per lane and instruction, no registers in
    // between.  Full tiles address memory as (uniform base of the tile's rows) + (this lane's fixed 32-bit
    // offset), which costs no vector arithmetic.  Tiles that reach past the end of the keys (prefix tail,
    // last tree tile) compute per-lane addresses and re-read the last valid row for the rows past the end:
    // their scores are masked below, so their probabilities are exactly zero and the values only need to be
    // finite.  Written as assembly on purpose: the compiler does not track these loads, so it puts no wait
    // between them and the LDS reads of the tile being computed; completion is awaited explicitly, per tile,
    // with s_waitcnt vmcnt (loads complete in order) ahead of the barrier that publishes the buffer.
    const unsigned kofs_p = (unsigned)(kkey0 * (int)a.kps[2] * ESZ + kcol), vofs_p = (unsigned)(kkey0 * (int)a.vps[2] * ESZ + vcol);
    const unsigned kofs_t = (unsigned)(kkey0 * (int)a.kts[2] * ESZ + kcol), vofs_t = (unsigned)(kkey0 * (int)a.vts[2] * ESZ + vcol);
    const int L = clamp_len(L_raw, a_max_prefix);
    const int ptiles = (L + TK - 1) / TK, ttiles = (a_nk + TK - 1) / TK;
    int t0, t1;
    split_range(ptiles + ttiles, a_splits, a_inv_splits, split, t0, t1);
    auto request_tile = [&](int t, auto buf_c) {
        const int buf = buf_c;                 // a compile-time constant or, in the wide variant's fast loop, a value
        const bool tree = t >= ptiles;
        // the mask word of a tree tile travels ahead of the tile's K/V (older, so it has landed when the tile's
        // wait is over)
        if (tree) {
            const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(s_mw + (buf * NWAVES + wave) * 128);
            const unsigned int* const wp = (const unsigned int*)(mask_row + (t - ptiles));
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_w), "v"(wp) : "m0", "memory");
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_w + 256), "v"(wp + 1) : "m0", "memory");
        }
        const int key0 = tree ? (t - ptiles) * TK : t * TK;
        const int last = (tree ? a_nk : L) - 1;
        const long long ks = (tree ? a.kts[2] : a.kps[2]) * ESZ;      // row strides in bytes
        const long long vs = (tree ? a.vts[2] : a.vps[2]) * ESZ;
        const unsigned char* kbase = tree ? kt : kp;
        const unsigned char* vbase = tree ? vt : vp;
        unsigned int* const lk = s_buf + buf * BUF;
        unsigned int* const lv = lk + TK * D / 2;
        if (key0 + TK - 1 <= last) {
            const unsigned kofs = tree ? kofs_t : kofs_p, vofs = tree ? vofs_t : vofs_p;
            const unsigned char* gk = kbase + (long long)key0 * ks;       // uniform: rows key0 + cc KSTEP of the tile
            const unsigned char* gv = vbase + (long long)key0 * vs;
            unsigned lds_k = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(lk + wave_u * 256);
            unsigned lds_v = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(lv + wave_u * 256);
#pragma unroll
            for (int cc = 0; cc < CH; ++cc) {                 // 16-byte slots cc * NT + wave * 64 + lane
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_k), "v"(kofs), "s"(gk) : "m0", "memory");
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_v), "v"(vofs), "s"(gv) : "m0", "memory");
                gk += KSTEP * ks; gv += KSTEP * vs;
                lds_k += NT * 16; lds_v += NT * 16;
            }
        } else {
#pragma unroll
            for (int cc = 0; cc < CH; ++cc) {
                const int slot0 = cc * NT + wave_u * 64;
                const unsigned lds_k = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(lk + slot0 * 4);
                const unsigned lds_v = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(lv + slot0 * 4);
                int row = key0 + kkey0 + cc * KSTEP;
                row = row < last ? row : last;
                const unsigned char* gk = kbase + row * ks + kcol;
                const unsigned char* gv = vbase + row * vs + vcol;
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_k), "v"(gk) : "m0", "memory");
                asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_v), "v"(gv) : "m0", "memory");
            }
        }
    };

    // KV8: widen the tile that has just landed in buffer `buf`, in place.  Every thread reads the sixteen-byte pieces
    // it owns (sixteen values each), the workgroup meets (the bf16 tile overwrites the bytes), the pieces are written
    // as bf16 where the operand reads expect them (K: 16-byte chunk c of row r at position c ^ (r mod 16); V: 32-byte
    // segment g at g ^ v_swizzle(r)), and the workgroup meets again.
    auto widen_tile = [&](int buf) {
        unsigned char* const rk = (unsigned char*)(s_buf + buf * BUF);
        unsigned char* const rv = rk + TK * D * 2;
        u32x4 wk[CH], wv[CH];
#pragma unroll
        for (int cc = 0; cc < CH; ++cc) {
            wk[cc] = *(const u32x4*)(rk + (cc * NT + tid) * 16);
            wv[cc] = *(const u32x4*)(rv + (cc * NT + tid) * 16);
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        auto widen = [](const u32x4& w, u32x4& lo, u32x4& hi) {
            unsigned int o[8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const auto p01 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);     // bytes 0, 1 of the word
                const auto p23 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);      // bytes 2, 3
                o[2 * i] = (__float_as_uint(p01[0]) >> 16) | (__float_as_uint(p01[1]) & 0xffff0000u);
                o[2 * i + 1] = (__float_as_uint(p23[0]) >> 16) | (__float_as_uint(p23[1]) & 0xffff0000u);
            }
            lo = u32x4{o[0], o[1], o[2], o[3]};
            hi = u32x4{o[4], o[5], o[6], o[7]};
        };
#pragma unroll
        for (int cc = 0; cc < CH; ++cc) {
            const int sigma = cc * NT + tid, row = sigma / CPRG, c16 = sigma % CPRG;
            u32x4 lo, hi;
            widen(wk[cc], lo, hi);
            unsigned short* const krow = (unsigned short*)rk + row * D;
            *(u32x4*)(krow + (((2 * c16) ^ (row & (CPR - 1))) << 3)) = lo;
            *(u32x4*)(krow + (((2 * c16 + 1) ^ (row & (CPR - 1))) << 3)) = hi;
            widen(wv[cc], lo, hi);
            unsigned short* const vseg = (unsigned short*)rv + row * D + ((c16 ^ v_swizzle(row)) << 4);
            *(u32x4*)vseg = lo;
            *(u32x4*)(vseg + 8) = hi;
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    };
    // The first PD tiles are requested at once.  A split with fewer tiles issues the same number of loads all the
    // same (one word each, into the unused buffer's mask-word slots: a load without a destination register): the
    // wait for Q below can then name a fixed count of younger requests.
    auto pad_requests = [&](int buf) {
        const unsigned lds_w = (unsigned)(size_t)(__attribute__((address_space(3))) void*)(s_mw + (buf * NWAVES + wave) * 128);
#pragma unroll
        for (int i = 0; i < LPT; ++i)
            asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_w), "v"(a_prefix_len) : "m0", "memory");
    };
    if (t0 < t1) request_tile(t0, std::integral_constant<int, 0>{}); else pad_requests(0);
    if (PD > 1) { if (t0 + 1 < t1) request_tile(t0 + 1, std::integral_constant<int, (PD > 1 ? 1 : 0)>{}); else pad_requests(1); }
    if (PD > 2) { if (t0 + 2 < t1) request_tile(t0 + 2, std::integral_constant<int, (PD > 2 ? 2 : 0)>{}); else pad_requests(2); }
    if (tid == 0 && hk == 0 && split == 0 && rb == 0) report_clamp(a.counters, L_raw, a_max_prefix);
    // Q has landed when at most the PD request groups issued behind it are outstanding (a tree tile's two mask
    // words are not counted: the wait is then on the safe side)
    wait_q<PD * LPT, SLABS>(qw);
    bf16x8 qf[SLABS];
#pragma unroll
    for (int s = 0; s < SLABS; ++s) qf[s] = __builtin_bit_cast(bf16x8, qw[s]);
    // One tile, out of buffer CUR.  The buffer index is a compile-time constant (the loop below is unrolled
    // NBUF times), so that every LDS address of the operand reads is a loop-invariant per-lane value plus an
    // immediate offset.
    auto tile_step = [&](int t, auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value;
        constexpr int PREV = (CUR + NBUF - 1) % NBUF;      // buffer of tile t - 1 (= of tile t + PD)
        // my requests for tile t have landed (younger ones may still be in flight); after the barrier
        // everybody's have, and everybody is done reading the buffer of tile t - 1
        // (a request group holds LPT tile loads, plus one mask word for a tree tile: allowing only
        // ahead * LPT younger loads to be outstanding is then on the safe side)
        const int ahead = t1 - 1 - t < PD - 1 ? t1 - 1 - t : PD - 1;
        if (ahead <= 0)      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(LPT) : "memory");
        else                 asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LPT) : "memory");
        if (t + PD < t1) request_tile(t + PD, std::integral_constant<int, PREV>{});
        if constexpr (KV8) widen_tile(CUR);

        const unsigned short* const s_k = (const unsigned short*)(s_buf + CUR * BUF);
        const unsigned short* const s_v = s_k + TK * D;

        const bool tree = t >= ptiles;
        const int key0 = tree ? (t - ptiles) * TK : t * TK;
        const int kend = tree ? a_nk : L;
        // visibility of the tile's 64 keys for this lane's query: keys that exist (a uniform bit run), and on
        // tree tiles the row's ancestor bits
        const bool masked = tree || key0 + TK > kend;
        uint64_t vis = kend - key0 >= TK ? ~0ull : ((1ull << (kend - key0)) - 1ull);
        if (tree) vis &= (uint64_t)s_mw[(CUR * NWAVES + wave) * 128 + lane] | ((uint64_t)s_mw[(CUR * NWAVES + wave) * 128 + 64 + lane] << 32);

        // one 32-key block at a time: S^T = K Q^T, online softmax, O^T += V^T P^T
#pragma unroll
        for (int j = 0; j < NKB; ++j) {
            const int kbi = WIDE ? j : kh;
            f32x16 sacc;
            u32x4 kfr[SLABS];
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
            for (int s = 0; s < SLABS; ++s) kfr[s] = *(const u32x4*)(s_k + (32 * kbi + l32) * D + (((2 * s) ^ kx) << 3));
#pragma unroll
            for (int s = 0; s < SLABS; ++s)
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfr[s]), qf[s], sacc, 0, 0, 0);
            // visibility; accumulator element v is key 32 kbi + 8 (v/4) + 4 h + v%4
            if (masked) {
                const unsigned int vw32 = (unsigned int)(kbi ? (vis >> 32) : vis) >> (4 * h);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // all ones if bit 8 (v/4) + v%4 is set, else zero; the score or -inf, chosen bit by bit
                    const unsigned int keep = (unsigned int)__builtin_amdgcn_sbfe((int)vw32, 8 * (v >> 2) + (v & 3), 1);
                    sacc[v] = __uint_as_float((__float_as_uint(sacc[v]) & keep) | (0xff800000u & ~keep));
                }
            }
            float tmax = sacc[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, sacc[v]);
            tmax = xhalf_max(tmax);
            const float m_new = fmaxf(m_run, tmax);
            bf16x8 pf[2];
            if (m_new == -INFINITY) {
#pragma unroll
                for (int v = 0; v < 16; ++v) pf[v >> 3][v & 7] = (__bf16)0.f;
            } else {
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);      // m_run = -inf gives 0
                const float mc = m_new * c;
                float psum = 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[v], c, -mc));
                    psum += p;
                    pf[v >> 3][v & 7] = (__bf16)p;
                }
                l_run = l_run * alpha + psum;
                m_run = m_new;
                if (__any(alpha != 1.f)) {       // the running maximum rarely moves after the first tiles
#pragma unroll
                    for (int d = 0; d < DB; ++d)
#pragma unroll
                        for (int v = 0; v < 16; ++v) oacc[d][v] *= alpha;
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
#pragma unroll
                for (int d = 0; d < DB; ++d) {
                    // this lane needs column 32d+l32 of keys 32kbi+16u+4h+{0..3} and of the same +8.
                    // Transpose load: lanes 4j..4j+3 of a 16-lane group address the 32-byte segment
                    // [key j][16 columns]; lane i of the group receives column i of the 4 keys.
                    const unsigned short* seg = s_v + (32 * kbi + 16 * u + 4 * h + tr_j) * D + (((2 * d) ^ vx) << 4) + tr_q;
                    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)seg);
                    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(seg + 8 * D));
                    const s16x8 vw = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vw), pf[u], oacc[d], 0, 0, 0);
                }
            }
        }
    };
    int t_done = t0;           // tiles [t0, t_done) are consumed
    if constexpr (WIDE) {
        // ---- fast loop of the 128-row variant over full prefix tiles: what the MFMA-bound shapes spend their time in.
        // The softmax reference of a row stays FIXED while scores do not exceed it by more than kSlack (in units
        // of log2 e / scale): p = 2^(c s - c ref) may then exceed one, which fp32 sums and bf16 operands take in
        // their stride, and O is never rescaled inside the loop -- the accumulators stay in their registers, the
        // loop body has no data-dependent path, and the two 32-key blocks of a tile are skewed against each other
        // so that the matrix pipe and the vector ALU work at the same time inside one wavefront (S of block 1
        // while the exponentials of block 0 are taken, P V of block 0 while those of block 1 are).  A score beyond
        // the slack (every row's first tile, then rarely) leaves the loop before anything of the tile is added;
        // the reference moves up, O and l are rescaled out here, and the loop is entered again at the same tile.
        constexpr float kSlack = 12.f;
#ifndef OT_ATTN_SUMCHECK
#define OT_ATTN_SUMCHECK 1
#endif
        constexpr float kSumLimit = 16.f * 4096.f;          // sixteen terms of at most 2^kSlack
        static_assert((NBUF & (NBUF - 1)) == 0, "the buffer of a tile is (t - t0) mod NBUF");
        // tile t has landed for this lane when only the requests of the tiles behind it are outstanding; after the
        // barrier it has for everybody, and everybody is done with the buffer that tile t + PD goes into
        auto stage_tile = [&](int t) {
            const int ahead = t1 - 1 - t < PD - 1 ? t1 - 1 - t : PD - 1;
            if (ahead <= 0)      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(LPT) : "memory");
            else                 asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LPT) : "memory");
            if (t + PD < t1) request_tile(t + PD, (t + PD - t0) & (NBUF - 1));
            if constexpr (KV8) widen_tile((t - t0) & (NBUF - 1));
        };
        const int t_full = min(t1, L / TK);                      // tiles below t_full are full prefix tiles
        auto kfrag = [&](const unsigned short* s_k, int kb, int s) {
            return *(const u32x4*)(s_k + (32 * kb + l32) * D + (((2 * s) ^ kx) << 3));
        };
        auto vfrag = [&](const unsigned short* s_v, int kb, int u, int d) {
            // column 32d+l32 of keys 32kb+16u+4h+{0..3} and of the same +8 (transpose loads, see tile_step)
            const unsigned short* seg = s_v + (32 * kb + 16 * u + 4 * h + tr_j) * D + (((2 * d) ^ vx) << 4) + tr_q;
            const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)seg);
            const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(seg + 8 * D));
            return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
        };
        auto row_max = [&](const f32x16& x) {                   // eight three-input maxima
            float m = fmaxf(fmaxf(x[0], x[1]), x[2]);
#pragma unroll
            for (int v = 3; v < 15; v += 2) m = fmaxf(fmaxf(m, x[v]), x[v + 1]);
            return xhalf_max(fmaxf(m, x[15]));
        };
        int t = t0;
        bool staged = false;                                      // tile t has been awaited and published
        float seen = -INFINITY;                                   // largest score of the tile that left the loop
        while (t < t_full) {
            if (!staged) {
                stage_tile(t);
                staged = true;
            }
            {   // move the reference up to what tile t needs; O and l follow
                const unsigned short* const s_k = (const unsigned short*)(s_buf + ((t - t0) & (NBUF - 1)) * BUF);
                f32x16 sa, sb;
#pragma unroll
                for (int v = 0; v < 16; ++v) { sa[v] = 0.f; sb[v] = 0.f; }
#pragma unroll
                for (int s = 0; s < SLABS; ++s) {
                    sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfrag(s_k, 0, s)), qf[s], sa, 0, 0, 0);
                    sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kfrag(s_k, 1, s)), qf[s], sb, 0, 0, 0);
                }
                const float m_new = fmaxf(m_run, fmaxf(row_max(sa), row_max(sb)));
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);      // m_run = -inf gives 0
                l_run *= alpha;
#pragma unroll
                for (int d = 0; d < DB; ++d)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[d][v] *= alpha;
                m_run = m_new;
            }
            const float mc = m_run * c;
            const float limit = m_run + kSlack / c;
            for (;;) {
                if (!staged) stage_tile(t);
                staged = true;
                const unsigned short* const s_k = (const unsigned short*)(s_buf + ((t - t0) & (NBUF - 1)) * BUF);
                const unsigned short* const s_v = s_k + TK * D;
                u32x4 kf[SLABS];
                bf16x8 va[2][DB], vb[2][DB];       // V operands of block 0 and of block 1
                f32x16 s0, s1;
#pragma unroll
                for (int s = 0; s < SLABS; ++s) kf[s] = kfrag(s_k, 0, s);
#pragma unroll
                for (int v = 0; v < 16; ++v) { s0[v] = 0.f; s1[v] = 0.f; }
#pragma unroll
                for (int s = 0; s < SLABS; ++s)
                    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s]), qf[s], s0, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < SLABS; ++s) kf[s] = kfrag(s_k, 1, s);
#if !OT_ATTN_SUMCHECK
                seen = row_max(s0);
                if (__any(seen > limit)) break;
#endif
                __builtin_amdgcn_sched_barrier(0);
                // S of block 1 in the matrix pipe, the exponentials of block 0 in the vector ALU, the V operands of
                // block 0 on their way.  One matrix instruction, then its share of the rest: the wavefront issues in
                // order, and a run of dependent MFMAs would otherwise hold everything else back until the last one.
#pragma unroll
                for (int s = 0; s < SLABS; ++s)
                    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s]), qf[s], s1, 0, 0, 0);
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int d = 0; d < DB; ++d) va[u][d] = vfrag(s_v, 0, u, d);
                bf16x8 p0[2], p1[2];
                float psum = 0.f;
                const bf16x2 ones2 = {(__bf16)1.f, (__bf16)1.f};
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    // a pair of probabilities, rounded to the MFMA's operand type, and their sum taken from the
                    // rounded pair with one dot-product instruction (l then matches what P V multiplies by)
                    const bf16x2 pr = {(__bf16)__builtin_amdgcn_exp2f(fmaf(s0[v], c, -mc)),
                                       (__bf16)__builtin_amdgcn_exp2f(fmaf(s0[v + 1], c, -mc))};
                    psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, psum, false);
                    p0[v >> 3][v & 7] = pr[0];
                    p0[v >> 3][(v & 7) + 1] = pr[1];
                }
                // (the empty statement is a use of P here: the compiler would otherwise move the exponentials behind
                // the test below, out of the shadow of the matrix instructions)
                asm volatile("" ::"v"(p0[0]), "v"(p0[1]), "v"(psum));
#pragma unroll
                for (int i = 0; i < SLABS; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 4 * DB / SLABS, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 48 / SLABS, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                seen = row_max(s1);
#if OT_ATTN_SUMCHECK
                // block 0 is tested on what its exponentials came to instead of on its scores: a probability beyond
                // 2^kSlack shows in the lane's sum (all terms are positive; an overflow gives +inf), which is there
                // anyway, while the maximum of sixteen scores costs a dozen instructions.  Nothing of the tile has
                // been added yet.  The bound is on the sum of sixteen terms, so single terms up to 2^kSlack pass
                // as before and a few somewhat larger ones may: the formats have the room.
                if (__any(seen > limit || psum > kSumLimit)) break;
#else
                if (__any(seen > limit)) break;
#endif
                __builtin_amdgcn_sched_barrier(0);
                // P V of block 0 in the matrix pipe, the exponentials of block 1 in the vector ALU, the V operands of
                // block 1 on their way
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int d = 0; d < DB; ++d) oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[u][d], p0[u], oacc[d], 0, 0, 0);
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int d = 0; d < DB; ++d) vb[u][d] = vfrag(s_v, 1, u, d);
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    // a pair of probabilities, rounded to the MFMA's operand type, and their sum taken from the
                    // rounded pair with one dot-product instruction (l then matches what P V multiplies by)
                    const bf16x2 pr = {(__bf16)__builtin_amdgcn_exp2f(fmaf(s1[v], c, -mc)),
                                       (__bf16)__builtin_amdgcn_exp2f(fmaf(s1[v + 1], c, -mc))};
                    psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, psum, false);
                    p1[v >> 3][v & 7] = pr[0];
                    p1[v >> 3][(v & 7) + 1] = pr[1];
                }
#pragma unroll
                for (int i = 0; i < 2 * DB; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 48 / (2 * DB), 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                l_run += psum;
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int d = 0; d < DB; ++d) oacc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[u][d], p1[u], oacc[d], 0, 0, 0);
                staged = false;
                if (++t >= t_full) break;
            }
        }
        (void)seen;
        t_done = t;
        // the remaining tiles (the prefix tail and the tree tiles) take the general path, whose buffer index is a
        // compile-time constant: tile t sits in buffer (t - t0) mod NBUF
        for (int tt = t_done; tt < t1; ++tt) {
            const int bi = (tt - t0) & (NBUF - 1);
            if (bi == 0)                   tile_step(tt, std::integral_constant<int, 0>{});
            else if (bi == 1)              tile_step(tt, std::integral_constant<int, 1>{});
            else if (NBUF > 2 && bi == 2)  tile_step(tt, std::integral_constant<int, (NBUF > 2 ? 2 : 0)>{});
            else if (NBUF > 3)             tile_step(tt, std::integral_constant<int, (NBUF > 3 ? 3 : 0)>{});
        }
    } else {
        for (int t = t0; t < t1; t += NBUF) {
            tile_step(t, std::integral_constant<int, 0>{});
            if (t + 1 < t1) tile_step(t + 1, std::integral_constant<int, 1>{});
            if (NBUF > 2 && t + 2 < t1) tile_step(t + 2, std::integral_constant<int, (NBUF > 2 ? 2 : 0)>{});
            if (NBUF > 3 && t + 3 < t1) tile_step(t + 3, std::integral_constant<int, (NBUF > 3 ? 3 : 0)>{});
        }
    }
    (void)t_done;

    l_run = xhalf_sum(l_run);
    if (!WIDE) {
        // merge the two key-half waves of each query block through LDS (all tiles are consumed)
        float* s_merge = (float*)s_buf;          // [2 qb][64 lanes][MST]
        float* mine = s_merge + (qb * 64 + lane) * MST;
        __syncthreads();
        if (kh == 1) {
#pragma unroll
            for (int d = 0; d < DB; ++d)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4)
                    *(f32x4*)(mine + d * 16 + 4 * v4) =
                        f32x4{oacc[d][4 * v4], oacc[d][4 * v4 + 1], oacc[d][4 * v4 + 2], oacc[d][4 * v4 + 3]};
            *(f32x4*)(mine + DB * 16) = f32x4{m_run, l_run, 0.f, 0.f};
        }
        __syncthreads();
        if (kh == 0) {
            const f32x4 ml2 = *(const f32x4*)(mine + DB * 16);
            const float m2 = ml2.x, l2 = ml2.y;
            const float mm = fmaxf(m_run, m2);
            float a1 = 0.f, a2 = 0.f;
            if (mm != -INFINITY) {
                a1 = __builtin_amdgcn_exp2f((m_run - mm) * c);
                a2 = __builtin_amdgcn_exp2f((m2 - mm) * c);
            }
            l_run = l_run * a1 + l2 * a2;
            m_run = mm;
#pragma unroll
            for (int d = 0; d < DB; ++d)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const f32x4 o2 = *(const f32x4*)(mine + d * 16 + 4 * v4);
                    oacc[d][4 * v4] = oacc[d][4 * v4] * a1 + o2.x * a2;
                    oacc[d][4 * v4 + 1] = oacc[d][4 * v4 + 1] * a1 + o2.y * a2;
                    oacc[d][4 * v4 + 2] = oacc[d][4 * v4 + 2] * a1 + o2.z * a2;
                    oacc[d][4 * v4 + 3] = oacc[d][4 * v4 + 3] * a1 + o2.w * a2;
                }
        }
    }
    const bool holder = WIDE || kh == 0;         // this wavefront holds finished (O, m, l) of its 32 rows

    if (a_splits == 1) {
        if (holder && row_ok) {
            const float inv = l_run > 0.f ? v_factor / l_run : 0.f;
            unsigned short* orow =
                (unsigned short*)a.O + (long long)b * a.os[0] + (long long)hq * a.os[1] + (long long)node * a.os[2];
#pragma unroll
            for (int d = 0; d < DB; ++d)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    unsigned short o4[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o4[e] = __builtin_bit_cast(unsigned short, (__bf16)(oacc[d][v4 * 4 + e] * inv));
                    uint2 pk;
                    pk.x = (unsigned)o4[0] | ((unsigned)o4[1] << 16);
                    pk.y = (unsigned)o4[2] | ((unsigned)o4[3] << 16);
                    *(uint2*)(orow + 32 * d + 8 * v4 + 4 * h) = pk;
                }
        }
        return;
    }

    // ---- several splits: leave the partial, take a ticket, the last one merges ----
    // Partials travel between workgroups (on different XCDs, each with its own L2) through device-scope
    // atomic stores and loads, which write through / read around the caches; a device-scope fence would
    // instead write back and invalidate the whole L2 once per workgroup.  Order: every wavefront waits
    // until its stores have completed (vmcnt), the workgroup meets at a barrier, then one thread takes the
    // ticket; the workgroup that sees the last ticket therefore reads completed partials only.
    // Only the live rows of a query block travel (a block holds live = min(32, g n - first row) of them):
    // part_o  [group][split][query block][e][64] x 8 bytes; e = (d block, group of four accumulator values as bf16)
    //         -- or (d block, pair of floats) when the exchange is fp32 -- and the live lanes of the two half-waves
    //         packed at the front of each 64-slot line (slot h live + l32): every store and load instruction touches
    //         one contiguous run, and nothing is moved for rows that do not exist
    // part_ml [group][split][query block][row] (m c, l) as two floats
    typedef unsigned long long u64;
    // EPS 64-bit elements per (lane, d block): pairs of floats, or with bf16 partials groups of four values
    constexpr int EPS = OT_ATTN_PART_BF16 ? 4 : 8;
    auto pack2 = [](float x, float y) -> u64 { return (u64)__float_as_uint(x) | ((u64)__float_as_uint(y) << 32); };
    auto pack4 = [](float x, float y, float z, float w) -> u64 {
        const bf16x2 lo = {(__bf16)x, (__bf16)y}, hi = {(__bf16)z, (__bf16)w};
        return (u64)__builtin_bit_cast(unsigned int, lo) | ((u64)__builtin_bit_cast(unsigned int, hi) << 32);
    };
    const int group = bz * a_row_blocks + rb;
    const int rows_all = a_g * n;
    if (holder && row_ok) {
        const int live = min(32, rows_all - (rb * ROWS + qb * 32));
        u64* po = (u64*)a.part_o + (((size_t)group * a_splits + split) * NQB + qb) * (DB * EPS * 64) + h * live + l32;
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
            for (int e = 0; e < EPS; ++e) {
                const u64 w = OT_ATTN_PART_BF16
                                  ? pack4(oacc[d][4 * e % 16], oacc[d][(4 * e + 1) % 16], oacc[d][(4 * e + 2) % 16], oacc[d][(4 * e + 3) % 16])
                                  : pack2(oacc[d][2 * e], oacc[d][2 * e + 1]);
                __hip_atomic_store(po + (d * EPS + e) * 64, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        if (h == 0)                                                  // lanes l and l + 32 hold the same row
            __hip_atomic_store((u64*)a.part_ml + (((size_t)group * a_splits + split) * NQB + qb) * 32 + l32,
                               pack2(m_run == -INFINITY ? -INFINITY : m_run * c /* log2 units */, l_run),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0)
        s_last = __hip_atomic_fetch_add(a.counters + group, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                         (unsigned)(a_splits - 1) ? 1 : 0;
    __syncthreads();
    if (!s_last) return;
    if (tid == 0) __hip_atomic_store(a.counters + group, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch

    // merge: thread = (query block cq, lane) x DC of the DB d blocks, same register order as above
    constexpr int DC = WIDE ? DB : DB / 2;
    const int cq = WIDE ? wave : (wave & 1);
    const int d0 = WIDE ? 0 : (wave >> 1) * DC;
    const int rho2 = rb * ROWS + cq * 32 + l32;
    if (rho2 >= rows_all) return;                      // no row behind this lane (no barrier follows)
    const int live2 = min(32, rows_all - (rb * ROWS + cq * 32));
    // CHUNK splits at a time: all their loads are issued before the first one is used (each is a trip to
    // memory), and the running maximum M is carried from chunk to chunk like in the main loop.  The narrow
    // variant has the whole register file of its SIMD and takes eight splits -- normally all -- in one trip.
    constexpr int MREGS = WIDE ? 64 : 96;
    constexpr int CHUNK = MREGS / (DC * EPS * 2) < 1 ? 1 : MREGS / (DC * EPS * 2);   // register budget
    const u64* mlp = (const u64*)a.part_ml + ((size_t)group * a_splits * NQB + cq) * 32 + l32;
    const u64* pp = (const u64*)a.part_o + ((size_t)group * a_splits * NQB + cq) * (DB * EPS * 64) + d0 * EPS * 64 +
                    h * live2 + l32;
    float M = -INFINITY, Ls = 0.f;
    f32x16 acc[DC];
#pragma unroll
    for (int d = 0; d < DC; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[d][v] = 0.f;
    for (int s0 = 0; s0 < a_splits; s0 += CHUNK) {
        u64 ml[CHUNK], x[CHUNK][DC * EPS];
#pragma unroll
        for (int i = 0; i < CHUNK; ++i) {
            const int si = s0 + i < a_splits ? s0 + i : a_splits - 1;      // past the end: a copy, weight 0
            ml[i] = __hip_atomic_load(mlp + (size_t)si * NQB * 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int i = 0; i < CHUNK; ++i) {
            const int si = s0 + i < a_splits ? s0 + i : a_splits - 1;
            const u64* ps = pp + (size_t)si * NQB * (DB * EPS * 64);
#pragma unroll
            for (int e = 0; e < DC * EPS; ++e)
                x[i][e] = __hip_atomic_load(ps + e * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        float mi[CHUNK], m_new = M;
#pragma unroll
        for (int i = 0; i < CHUNK; ++i) {
            mi[i] = s0 + i < a_splits ? __uint_as_float((unsigned)ml[i]) : -INFINITY;
            m_new = fmaxf(m_new, mi[i]);
        }
        if (m_new == -INFINITY) continue;                                    // nothing visible so far
        const float alpha = __builtin_amdgcn_exp2f(M - m_new);                // M = -inf gives 0
        Ls *= alpha;
#pragma unroll
        for (int d = 0; d < DC; ++d)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[d][v] *= alpha;
#pragma unroll
        for (int i = 0; i < CHUNK; ++i) {
            const float w = mi[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mi[i] - m_new);
            Ls = fmaf(w, __uint_as_float((unsigned)(ml[i] >> 32)), Ls);
#pragma unroll
            for (int e = 0; e < DC * EPS; ++e) {
                const unsigned int lo = (unsigned)x[i][e], hi = (unsigned)(x[i][e] >> 32);
                if (OT_ATTN_PART_BF16) {
                    const int dd = e / EPS, v0 = 4 * (e % EPS);
                    acc[dd][v0] = fmaf(w, __uint_as_float(lo << 16), acc[dd][v0]);
                    acc[dd][v0 + 1] = fmaf(w, __uint_as_float(lo & 0xffff0000u), acc[dd][v0 + 1]);
                    acc[dd][v0 + 2] = fmaf(w, __uint_as_float(hi << 16), acc[dd][v0 + 2]);
                    acc[dd][v0 + 3] = fmaf(w, __uint_as_float(hi & 0xffff0000u), acc[dd][v0 + 3]);
                } else {
                    acc[e >> 3][2 * (e & 7)] = fmaf(w, __uint_as_float(lo), acc[e >> 3][2 * (e & 7)]);
                    acc[e >> 3][2 * (e & 7) + 1] = fmaf(w, __uint_as_float(hi), acc[e >> 3][2 * (e & 7) + 1]);
                }
            }
        }
        M = m_new;
    }
    {
        const int head2 = fast_div(rho2, n, a_inv_n);
        const int hq2 = hk * a_g + head2, node2 = rho2 - head2 * n;
        const float inv = Ls > 0.f ? v_factor / Ls : 0.f;
        unsigned short* orow =
            (unsigned short*)a.O + (long long)b * a.os[0] + (long long)hq2 * a.os[1] + (long long)node2 * a.os[2];
#pragma unroll
        for (int d = 0; d < DC; ++d)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                unsigned short o4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o4[e] = __builtin_bit_cast(unsigned short, (__bf16)(acc[d][v4 * 4 + e] * inv));
                uint2 pk;
                pk.x = (unsigned)o4[0] | ((unsigned)o4[1] << 16);
                pk.y = (unsigned)o4[2] | ((unsigned)o4[3] << 16);
                *(uint2*)(orow + 32 * (d0 + d) + 8 * v4 + 4 * h) = pk;
            }
    }
}

// ---------------------------------------------------------------------------
// f32 kernel: 16 query rows of one query head x 32-key tiles, fp32 FMA arithmetic
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnKArgs a) {
    constexpr int TK = 32, RB = 16;
    constexpr int KPAD = D + 4;
    constexpr int EPT = D / 16;            // output columns per thread
    __shared__ __attribute__((aligned(16))) float s_q[RB * D];
    __shared__ __attribute__((aligned(16))) float s_k[TK * KPAD];
    __shared__ __attribute__((aligned(16))) float s_v[TK * D];
    __shared__ float s_p[RB * TK];

    const int tid = threadIdx.x, r = tid >> 4, c = tid & 15;
    const int split = blockIdx.x, rb = blockIdx.y;
    const int b = blockIdx.z / a.q_heads, hq = blockIdx.z - b * a.q_heads;
    const int hk = hq / a.g;
    const int n = a.n;
    const int L = clamp_len(a.prefix_len[b], a.max_prefix);
    if (tid == 0 && hq == 0 && split == 0 && rb == 0) report_clamp(a.counters, a.prefix_len[b], a.max_prefix);
    const int ptiles = (L + TK - 1) / TK, ttiles = (a.nk + TK - 1) / TK;
    int t0, t1;
    split_range(ptiles + ttiles, a.splits, a.inv_splits, split, t0, t1);
    const int node = rb * RB + r;
    const bool row_ok = node < n;

    const float* qbase = (const float*)a.Q + (long long)b * a.qs[0] + (long long)hq * a.qs[1];
    for (int i = tid; i < RB * D / 4; i += 256) {
        const int rr = i / (D / 4), cc = (i % (D / 4)) * 4;
        f32x4 w = {0.f, 0.f, 0.f, 0.f};
        if (rb * RB + rr < n) w = *(const f32x4*)(qbase + (long long)(rb * RB + rr) * a.qs[2] + cc);
        *(f32x4*)(s_q + rr * D + cc) = w;
    }
    // this row's ancestor mask: the 64-bit word that covers a 32-key tree tile is read with the tile
    const uint64_t* const mask_row = a.mask + ((long long)b * n + (row_ok ? node : 0)) * a.W;

    const float* kp = (const float*)a.Kp + (long long)b * a.kps[0] + (long long)hk * a.kps[1];
    const float* vp = (const float*)a.Vp + (long long)b * a.vps[0] + (long long)hk * a.vps[1];
    const float* kt = (const float*)a.Kt + (long long)b * a.kts[0] + (long long)hk * a.kts[1];
    const float* vt = (const float*)a.Vt + (long long)b * a.vts[0] + (long long)hk * a.vts[1];

    float m_run = -INFINITY, l_run = 0.f;
    float o[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) o[e] = 0.f;

    for (int t = t0; t < t1; ++t) {
        const bool tree = t >= ptiles;
        const int key0 = tree ? (t - ptiles) * TK : t * TK;
        const int kend = tree ? a.nk : L;
        const float* kb = tree ? kt : kp;
        const float* vb = tree ? vt : vp;
        const long long ks = tree ? a.kts[2] : a.kps[2];
        const long long vs = tree ? a.vts[2] : a.vps[2];
        __syncthreads();
        const uint64_t mword = (tree && row_ok) ? mask_row[key0 >> 6] : 0ull;
        for (int i = tid; i < TK * D / 4; i += 256) {
            const int key = i / (D / 4), cc = (i % (D / 4)) * 4;
            f32x4 kw = {0.f, 0.f, 0.f, 0.f}, vw = {0.f, 0.f, 0.f, 0.f};
            if (key0 + key < kend) {
                kw = *(const f32x4*)(kb + (long long)(key0 + key) * ks + cc);
                vw = *(const f32x4*)(vb + (long long)(key0 + key) * vs + cc);
            }
            *(f32x4*)(s_k + key * KPAD + cc) = kw;
            *(f32x4*)(s_v + key * D + cc) = vw;
        }
        __syncthreads();
        float s2[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int kl = c + 16 * u;
            float acc = 0.f;
#pragma unroll 8
            for (int d = 0; d < D; d += 4) {
                const f32x4 qv = *(const f32x4*)(s_q + r * D + d);
                const f32x4 kv = *(const f32x4*)(s_k + kl * KPAD + d);
                acc = fmaf(qv.x, kv.x, acc); acc = fmaf(qv.y, kv.y, acc);
                acc = fmaf(qv.z, kv.z, acc); acc = fmaf(qv.w, kv.w, acc);
            }
            const int key = key0 + kl;
            bool ok = row_ok && key < kend;
            if (tree) ok = ok && ((mword >> (key & 63)) & 1ull);
            s2[u] = ok ? acc * a.scale_log2 : -INFINITY;
        }
        const float tmax = row16_max(fmaxf(s2[0], s2[1]));
        const float m_new = fmaxf(m_run, tmax);
        float alpha = 1.f, p0 = 0.f, p1 = 0.f;
        if (m_new != -INFINITY) {
            alpha = exp2f(m_run - m_new);
            p0 = exp2f(s2[0] - m_new);
            p1 = exp2f(s2[1] - m_new);
            m_run = m_new;
        }
        s_p[r * TK + c] = p0;
        s_p[r * TK + c + 16] = p1;
        __syncthreads();
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < EPT; ++e) o[e] *= alpha;
        for (int jj = 0; jj < TK; ++jj) {
            const float p = s_p[r * TK + jj];
            psum += p;
#pragma unroll
            for (int e = 0; e < EPT; ++e) o[e] = fmaf(p, s_v[jj * D + c + 16 * e], o[e]);
        }
        l_run = l_run * alpha + psum;
    }
    if (!row_ok) return;
    const long long row = ((long long)b * a.q_heads + hq) * n + node;
    if (a.splits == 1) {
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
        float* orow = (float*)a.O + (long long)b * a.os[0] + (long long)hq * a.os[1] + (long long)node * a.os[2];
#pragma unroll
        for (int e = 0; e < EPT; ++e) orow[c + 16 * e] = o[e] * inv;
    } else {
        float* po = a.part_o + (row * a.splits + split) * D;
#pragma unroll
        for (int e = 0; e < EPT; ++e) po[c + 16 * e] = o[e];
        if (c == 0) {
            a.part_ml[(row * a.splits + split) * 2] = m_run;
            a.part_ml[(row * a.splits + split) * 2 + 1] = l_run;
        }
    }
}

// f32 path only (the bf16 kernel merges its own partials).
// Merge the per-split partials of one output row: O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// One wavefront per row (4 rows per workgroup); lane s holds split s's (m, l), the weights are
// broadcast with v_readlane, every lane accumulates D/64 columns.
__global__ __launch_bounds__(256) void attn_combine_kernel(const AttnKArgs a) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long rows = (long long)a.batch * a.q_heads * a.n;
    if (row >= rows) return;
    const int n = a.n;
    const int node = (int)(row % n);
    const int hq = (int)((row / n) % a.q_heads);
    const int b = (int)(row / ((long long)n * a.q_heads));
    const float* ml = a.part_ml + row * a.splits * 2;
    const float* po = a.part_o + row * a.splits * a.D;
    float m = -INFINITY, l = 0.f;
    if (lane < a.splits) { m = ml[2 * lane]; l = ml[2 * lane + 1]; }
    const float M = wave_max_f(m);
    const float w = (m == -INFINITY) ? 0.f : exp2f(m - M);
    float wl = w * l;
    wl += __int_as_float(dpp_i<DPP_QUAD_XOR1>(0, __float_as_int(wl)));
    wl += __int_as_float(dpp_i<DPP_QUAD_XOR2>(0, __float_as_int(wl)));
    wl += __int_as_float(dpp_i<DPP_ROW_HALF_MIRROR>(0, __float_as_int(wl)));
    wl += __int_as_float(dpp_i<DPP_ROW_MIRROR>(0, __float_as_int(wl)));
    const float Lsum = (rl_f(wl, 0) + rl_f(wl, 16)) + (rl_f(wl, 32) + rl_f(wl, 48));
    const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
    const int per = a.D / 64;                 // 1 or 2 columns per lane
    float acc0 = 0.f, acc1 = 0.f;
    for (int s = 0; s < a.splits; ++s) {
        const float ws = rl_f(w, s);
        if (per == 2) {
            const float2 v = *(const float2*)(po + (long long)s * a.D + 2 * lane);
            acc0 = fmaf(ws, v.x, acc0); acc1 = fmaf(ws, v.y, acc1);
        } else {
            acc0 = fmaf(ws, po[(long long)s * a.D + lane], acc0);
        }
    }
    const long long off = (long long)b * a.os[0] + (long long)hq * a.os[1] + (long long)node * a.os[2] + per * lane;
    if (a.dtype == OT_BF16) {
        unsigned short* o = (unsigned short*)a.O + off;
        o[0] = __builtin_bit_cast(unsigned short, (__bf16)(acc0 * inv));
        if (per == 2) o[1] = __builtin_bit_cast(unsigned short, (__bf16)(acc1 * inv));
    } else {
        float* o = (float*)a.O + off;
        o[0] = acc0 * inv;
        if (per == 2) o[1] = acc1 * inv;
    }
}

__global__ void attn_clear_sync_kernel(unsigned int* p) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < OT_ATTN_SYNC_BYTES / 4) p[i] = 0u;
}

}  // namespace

static size_t align_up(size_t v, size_t al) { return (v + al - 1) / al * al; }

// Workgroups that the split count of the bf16 path aims at: what the chip holds at once (256 compute
// units; the narrow variant's three tile buffers allow one workgroup per unit at head_dim 128, the wide
// variant's two buffers allow two).
#ifndef OT_ATTN_NARROW_WGS
#define OT_ATTN_NARROW_WGS 256
#endif
#ifndef OT_ATTN_WIDE_WGS
#define OT_ATTN_WIDE_WGS 512
#endif

// Packed query rows per workgroup of the bf16 kernel: 64 (narrow: the wavefronts split each tile's keys), 128, or
// 256 when a KV head has more rows than that -- eight wavefronts then share every staged K/V tile, which halves the
// traffic into LDS per MFMA and leaves room for a ring of four tiles (three in flight).
// Batches take their jobs longest first (1) or in the order of their sequences (0).
#ifndef OT_ATTN_BALANCE
#define OT_ATTN_BALANCE 1
#endif
#ifndef OT_ATTN_ROWS256_FROM
#define OT_ATTN_ROWS256_FROM 129
#endif
static int attn_rows_per_workgroup(int rows_per_kv_head) {
    return rows_per_kv_head <= 64 ? 64 : (rows_per_kv_head >= OT_ATTN_ROWS256_FROM ? 256 : 128);
}

AttnPlan plan_attention(const ot_attn_params& p, bool kv8) {
    AttnPlan pl;
    pl.balance = 0;
    const int g = p.q_heads / p.kv_heads;
    int base, tile, rows_wg = 0, splits;
    if (p.dtype == OT_BF16) {
        const bool wide = g * p.n > 64;                    // wide variants when one KV head has more than 64 rows
        rows_wg = attn_rows_per_workgroup(g * p.n);
        if (kv8 && rows_wg == 256) rows_wg = 128;
        pl.row_blocks = (g * p.n + rows_wg - 1) / rows_wg;
        base = p.batch * p.kv_heads * pl.row_blocks;
        tile = 64;
        int target = wide ? (rows_wg == 256 ? OT_ATTN_WIDE_WGS / 2 : OT_ATTN_WIDE_WGS) : OT_ATTN_NARROW_WGS;
        if (!wide && p.head_dim == 64) target *= 2;
        splits = target / base;                            // never more workgroups than fit at once
        // A batch that fills the chip with one key range per (sequence, KV head): the lengths are known on the
        // device only, where the workgroups take their jobs longest first (see the kernel).  Measured: 3 % faster on
        // ragged batches of one and a half to three rounds of workgroups; from four rounds on the rounds even the
        // lengths out by themselves and the ranking's extra trip to memory per workgroup costs 1 %.
        if (OT_ATTN_BALANCE && wide && p.batch > 1 && p.batch <= 64 && splits <= 1 && base < 4 * target) pl.balance = 1;
    } else {
        pl.row_blocks = (p.n + 15) / 16;
        base = p.batch * p.q_heads * pl.row_blocks;
        tile = 32;
        splits = (512 + base - 1) / base;
    }
    const int nk = p.n_keys > 0 ? p.n_keys : p.n;
    const int max_tiles = (p.max_prefix + tile - 1) / tile + (nk + tile - 1) / tile;
    if (splits > max_tiles) splits = max_tiles;
    if (splits > kMaxSplits) splits = kMaxSplits;
    if (splits < 1) splits = 1;
#ifndef OT_ATTN_EVEN_OUT
#define OT_ATTN_EVEN_OUT 1
#endif
    if (OT_ATTN_EVEN_OUT) {
        // even out: every split gets the same number of tiles (the last one possibly fewer)
        const int per = (max_tiles + splits - 1) / splits;
        splits = (max_tiles + per - 1) / per;
    }
    pl.splits = splits;
    // bf16: partials are stored per workgroup (rows padded to the row block); f32: per output row
    const size_t rows = p.dtype == OT_BF16 ? (size_t)base * rows_wg : (size_t)p.batch * p.q_heads * p.n;
    const size_t part_elem = (p.dtype == OT_BF16 && OT_ATTN_PART_BF16) ? 2 : 4;
    pl.part_o_bytes = splits > 1 ? align_up(rows * splits * p.head_dim * part_elem, 256) : 0;
    pl.part_ml_bytes = splits > 1 ? align_up(rows * splits * 2 * 4, 256) : 0;
    pl.bytes = OT_ATTN_SYNC_BYTES + pl.part_o_bytes + pl.part_ml_bytes + 256;
    return pl;
}

int launch_tree_attention(const ot_attn_params& p, const AttnPlan& plan, const void* Q, const void* Kp, const void* Vp,
                          const void* Kt, const void* Vt, const int32_t* prefix_len, const uint64_t* mask, void* O,
                          void* workspace, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1, const float* k_scale,
                          const float* v_scale) {
    const bool kv8 = k_scale != nullptr;
    AttnKArgs a;
    a.splits_share_xcd = 0;
    a.Q = Q; a.Kp = Kp; a.Vp = Vp; a.Kt = Kt; a.Vt = Vt;
    a.prefix_len = prefix_len; a.mask = mask; a.O = O;
    a.k_scale = k_scale; a.v_scale = v_scale;
    a.counters = (unsigned int*)workspace;
    a.part_o = (float*)((char*)workspace + OT_ATTN_SYNC_BYTES);
    a.part_ml = (float*)((char*)workspace + OT_ATTN_SYNC_BYTES + plan.part_o_bytes);
    a.batch = p.batch; a.q_heads = p.q_heads; a.kv_heads = p.kv_heads; a.g = p.q_heads / p.kv_heads;
    a.n = p.n; a.nk = p.n_keys > 0 ? p.n_keys : p.n; a.D = p.head_dim; a.max_prefix = p.max_prefix; a.splits = plan.splits;
    a.W = OT_MASK_WORDS(a.nk); a.dtype = p.dtype;
    const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
    a.scale_log2 = scale * kLog2e;
    for (int i = 0; i < 3; ++i) {
        a.qs[i] = p.q_strides[i]; a.kps[i] = p.kp_strides[i]; a.vps[i] = p.vp_strides[i];
        a.kts[i] = p.kt_strides[i]; a.vts[i] = p.vt_strides[i]; a.os[i] = p.o_strides[i];
    }
    a.row_blocks = plan.row_blocks;
    auto magic = [](int d) { return d <= 1 ? 0u : (unsigned int)((0x100000000ull + (unsigned)d - 1) / (unsigned)d); };
    a.inv_splits = magic(a.splits); a.inv_kv_heads = magic(a.kv_heads); a.inv_n = magic(a.n);
    if (p.dtype == OT_BF16) {
        int rows_wg = attn_rows_per_workgroup(a.g * p.n);
        if (kv8 && rows_wg == 256) rows_wg = 128;
        const long long units = (long long)p.batch * p.kv_heads * plan.splits;
        const long long unit_groups = (units + 7) / 8;      // the same count either way when pairs % 8 == 0
        a.splits_share_xcd = (!plan.balance && plan.splits > 1 && ((long long)p.batch * p.kv_heads) % 8 == 0) ? 1 : 0;
        if (unit_groups > 65535 || 8LL * plan.row_blocks > 0x7fffffffLL) return OT_ERR_UNSUPPORTED;   // cannot happen within the limits
        if (plan.splits > 1 && (long long)p.batch * p.kv_heads * plan.row_blocks * 4 > OT_ATTN_STATUS_OFFSET)
            return OT_ERR_UNSUPPORTED;      // cannot happen: splits > 1 only with few workgroups
        const dim3 grid((unsigned)(8 * plan.row_blocks), (unsigned)unit_groups);
#define OT_ATTN_ARGS a.prefix_len, a.mask, a.Q, a.splits, a.inv_splits, a.kv_heads, a.inv_kv_heads, a.n, a.inv_n, a
#define OT_ATTN_LAUNCH(DD, VV, K8, BB)                                                                       \
    do {                                                                                                   \
        const int nbuf = (VV) == 2 ? 4 : ((VV) == 1 ? 2 : OT_ATTN_NBUF_NARROW), nwaves = (VV) == 2 ? 8 : 4; \
        const size_t lds = (size_t)nbuf * (64 * DD + nwaves * 128) * sizeof(unsigned int);                 \
        if (lds > 64 * 1024)                                                                               \
            OT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_mfma_kernel<DD, VV, K8, BB>,                 \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));       \
        if (ev0 || ev1) hipExtLaunchKernelGGL((attn_mfma_kernel<DD, VV, K8, BB>), grid, dim3(64 * nwaves), lds, s, ev0, ev1, 0, OT_ATTN_ARGS); \
        else hipLaunchKernelGGL((attn_mfma_kernel<DD, VV, K8, BB>), grid, dim3(64 * nwaves), lds, s, OT_ATTN_ARGS); \
    } while (0)
        const int var = rows_wg == 256 ? 2 : (rows_wg == 128 ? 1 : 0);
        // (the 8-bit cache runs the 64- and 128-row variants; only wide variants take their jobs longest first)
#define OT_ATTN_PICK(DD, K8)                                                                                \
    do {                                                                                                    \
        if (var == 2 && !(K8)) { if (plan.balance) OT_ATTN_LAUNCH(DD, ((K8) ? 1 : 2), K8, true); else OT_ATTN_LAUNCH(DD, ((K8) ? 1 : 2), K8, false); } \
        else if (var >= 1)     { if (plan.balance) OT_ATTN_LAUNCH(DD, 1, K8, true); else OT_ATTN_LAUNCH(DD, 1, K8, false); } \
        else                   OT_ATTN_LAUNCH(DD, 0, K8, false);                                            \
    } while (0)
        if (kv8) { if (p.head_dim == 128) OT_ATTN_PICK(128, true); else OT_ATTN_PICK(64, true); }
        else     { if (p.head_dim == 128) OT_ATTN_PICK(128, false); else OT_ATTN_PICK(64, false); }
#undef OT_ATTN_PICK
#undef OT_ATTN_LAUNCH
#undef OT_ATTN_ARGS
    } else {
        const dim3 grid(plan.splits, plan.row_blocks, p.batch * p.q_heads);
        if (ev0 || ev1) {
            if (p.head_dim == 128) hipExtLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, s, ev0, ev1, 0, a);
            else                   hipExtLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, s, ev0, ev1, 0, a);
        } else {
            if (p.head_dim == 128) hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(256), 0, s, a);
            else                   hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(256), 0, s, a);
        }
    }
    OT_HIP_CHECK(hipGetLastError());
    if (plan.splits > 1 && p.dtype != OT_BF16) {
        const long long rows = (long long)p.batch * p.q_heads * p.n;
        hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a);
        OT_HIP_CHECK(hipGetLastError());
    }
    return OT_OK;
}

}  // namespace ot

using namespace ot;

static int validate_attn(const ot_attn_params* p, bool kv8 = false) {
    if (!p) return OT_ERR_INVALID_ARG;
    if (p->batch < 1 || p->q_heads < 1 || p->kv_heads < 1 || p->n < 1 || p->max_prefix < 0) return OT_ERR_INVALID_ARG;
    if (p->q_heads % p->kv_heads) return OT_ERR_INVALID_ARG;
    if (p->dtype != OT_F32 && p->dtype != OT_BF16) return OT_ERR_INVALID_ARG;
    if (!(p->softmax_scale >= 0.f)) return OT_ERR_INVALID_ARG;
    if (p->head_dim != 64 && p->head_dim != 128) return OT_ERR_UNSUPPORTED;
    if (p->n > OT_MAX_NODES) return OT_ERR_UNSUPPORTED;
    if (p->n_keys < 0) return OT_ERR_INVALID_ARG;
    if (p->n_keys > OT_MAX_TREE_KEYS) return OT_ERR_UNSUPPORTED;
    if ((long long)p->batch * p->q_heads > 65535 || (long long)p->batch * p->q_heads * p->n > 0x7fffffffLL)
        return OT_ERR_UNSUPPORTED;
    if (kv8 && p->dtype != OT_BF16) return OT_ERR_INVALID_ARG;      // Q and O of the 8-bit cache variant are bf16
    const int64_t* st[6] = {p->q_strides, p->kp_strides, p->vp_strides, p->kt_strides, p->vt_strides, p->o_strides};
    for (int t = 0; t < 6; ++t) {
        const int vec = (kv8 && t >= 1 && t <= 4) ? 16 : (p->dtype == OT_BF16 ? 8 : 4);      // elements per 16 bytes
        for (int i = 0; i < 3; ++i)
            if (st[t][i] < 0 || st[t][i] % vec) return OT_ERR_INVALID_ARG;
        if (st[t][2] < p->head_dim) return OT_ERR_INVALID_ARG;
        if (st[t][2] > (1 << 22)) return OT_ERR_UNSUPPORTED;    // 64 rows of a tile are addressed with 32-bit offsets
    }
    return OT_OK;
}

extern "C" {

size_t ot_attn_workspace_bytes(const ot_attn_params* p) {
    if (validate_attn(p) != OT_OK) return 0;
    const size_t plain = plan_attention(*p).bytes;
    // one workspace serves the 8-bit cache variant too, whose row blocks and key splits may differ
    const size_t kv8 = p->dtype == OT_BF16 ? plan_attention(*p, true).bytes : 0;
    return plain > kv8 ? plain : kv8;
}

static int attention_entry(const ot_attn_params* p, const void* Q, const void* K_prefix, const void* V_prefix,
                           const void* K_tree, const void* V_tree, const int32_t* prefix_len, const uint64_t* mask,
                           void* O, void* workspace, size_t workspace_bytes, void* hip_stream, void* ev0, void* ev1,
                           const float* k_scale = nullptr, const float* v_scale = nullptr, bool kv8 = false) {
    int st = validate_attn(p, kv8);
    if (st != OT_OK) return st;
    if (kv8 && (!k_scale || !v_scale || ((uintptr_t)k_scale % 4) || ((uintptr_t)v_scale % 4))) return OT_ERR_INVALID_ARG;
    if (!Q || !K_tree || !V_tree || !prefix_len || !mask || !O || !workspace) return OT_ERR_INVALID_ARG;
    if (p->max_prefix > 0 && (!K_prefix || !V_prefix)) return OT_ERR_INVALID_ARG;
    const void* ptrs[7] = {Q, K_prefix, V_prefix, K_tree, V_tree, O, workspace};
    for (int i = 0; i < 7; ++i)
        if (ptrs[i] && ((uintptr_t)ptrs[i] % 16)) return OT_ERR_INVALID_ARG;
    if (((uintptr_t)prefix_len % 4) || ((uintptr_t)mask % 8)) return OT_ERR_INVALID_ARG;
    const AttnPlan plan = plan_attention(*p, kv8);
    if (workspace_bytes < plan.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    return launch_tree_attention(*p, plan, Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, O, workspace,
                                 (hipStream_t)hip_stream, (hipEvent_t)ev0, (hipEvent_t)ev1, kv8 ? k_scale : nullptr,
                                 kv8 ? v_scale : nullptr);
}

int ot_attn_workspace_prepare(void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!workspace || ((uintptr_t)workspace % 16)) return OT_ERR_INVALID_ARG;
    if (workspace_bytes < OT_ATTN_SYNC_BYTES) return OT_ERR_WORKSPACE_TOO_SMALL;
    hipLaunchKernelGGL(attn_clear_sync_kernel, dim3(OT_ATTN_SYNC_BYTES / 4 / 256), dim3(256), 0, (hipStream_t)hip_stream,
                       (unsigned int*)workspace);
    OT_HIP_CHECK(hipGetLastError());
    return OT_OK;
}

int ot_tree_verify_attention(const ot_attn_params* p, const void* Q, const void* K_prefix, const void* V_prefix,
                             const void* K_tree, const void* V_tree, const int32_t* prefix_len, const uint64_t* mask,
                             void* O, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return attention_entry(p, Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, O, workspace, workspace_bytes,
                           hip_stream, nullptr, nullptr);
}

// ---------------------------------------------------------------------------
// Entry point for callers that cannot allocate: the workspace (ticket counters, status word, split partials) is a
// library-owned array in device memory.  Every GPU holds its own copy at its own address; host code never uses
// the array's name except to look that address up, once per device.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[OT_ATTN_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];       // device address of `scratch` on device i, null until looked up
}  // namespace

int ot_tree_verify_attention_noalloc(const ot_attn_params* p, const void* Q, const void* K_prefix, const void* V_prefix,
                                     const void* K_tree, const void* V_tree, const int32_t* prefix_len,
                                     const uint64_t* mask, void* O, void* hip_stream) {
    int st = validate_attn(p);
    if (st != OT_OK) return st;
    if (ot_attn_workspace_bytes(p) > (size_t)OT_ATTN_SCRATCH_BYTES) return OT_ERR_SCRATCH_LIMIT;
    int dev = -1;
    OT_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return OT_ERR_UNSUPPORTED;
    void* ptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            // set-up, once per device, with that device current: the address of this device's copy of the array,
            // and its ticket counters and status word cleared (by a kernel, which a graph capture could record)
            void* found = nullptr;
            OT_HIP_CHECK(hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)));
            if (!found || ((uintptr_t)found % 256)) return OT_ERR_HIP;
            hipLaunchKernelGGL(attn_clear_sync_kernel, dim3(OT_ATTN_SYNC_BYTES / 4 / 256), dim3(256), 0,
                               (hipStream_t)hip_stream, (unsigned int*)found);
            OT_HIP_CHECK(hipGetLastError());
            g_scratch_ptr[dev] = found;
        }
        ptr = g_scratch_ptr[dev];
    }
    return attention_entry(p, Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, O, ptr, OT_ATTN_SCRATCH_BYTES,
                           hip_stream, nullptr, nullptr);
}

int ot_tree_verify_attention_fp8kv(const ot_attn_params* p, const void* Q, const void* K_prefix, const void* V_prefix,
                                   const void* K_tree, const void* V_tree, const float* k_scale, const float* v_scale,
                                   const int32_t* prefix_len, const uint64_t* mask, void* O, void* workspace,
                                   size_t workspace_bytes, void* hip_stream) {
    return attention_entry(p, Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, O, workspace, workspace_bytes,
                           hip_stream, nullptr, nullptr, k_scale, v_scale, true);
}

int ot_tree_verify_attention_timed(const ot_attn_params* p, const void* Q, const void* K_prefix, const void* V_prefix,
                                   const void* K_tree, const void* V_tree, const int32_t* prefix_len,
                                   const uint64_t* mask, void* O, void* workspace, size_t workspace_bytes,
                                   void* hip_stream, void* kernel_begin_event, void* kernel_end_event) {
    return attention_entry(p, Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, O, workspace, workspace_bytes,
                           hip_stream, kernel_begin_event, kernel_end_event);
}

}  // extern "C"
