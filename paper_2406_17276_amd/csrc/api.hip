// C ABI of libopttree: argument validation, workspace carving and kernel sequencing.
// No arithmetic of the method lives here.
#include <string.h>

#include "common.hpp"

namespace ot {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

Frontier make_frontier(int k, int n, int depth) {
    Frontier f;
    memset(&f, 0, sizeof(f));
    f.F[0] = 1;
    f.row_start[0] = 0;
    long long rows = 0, pool = 0;
    for (int t = 0; t < depth; ++t) {
        rows += f.F[t];
        f.row_start[t + 1] = (int)rows;
        const long long next = (long long)k * f.F[t];
        f.F[t + 1] = (int)(next < n ? next : n);
        pool += f.F[t + 1];
    }
    f.rows = (int)rows;
    f.pool = (int)pool;
    return f;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static int validate_build(const ot_build_params* p, bool check_strides) {
    if (!p) return OT_ERR_INVALID_ARG;
    if (p->batch < 1 || p->vocab < 1 || p->depth < 1 || p->k < 1 || p->n < 1) return OT_ERR_INVALID_ARG;
    if (p->k > p->vocab) return OT_ERR_INVALID_ARG;
    if (p->logits_dtype != OT_F32 && p->logits_dtype != OT_BF16) return OT_ERR_INVALID_ARG;
    if (p->k > OT_MAX_TOPK || p->n > OT_MAX_NODES || p->depth > OT_MAX_DEPTH) return OT_ERR_UNSUPPORTED;
    if (scan_parts(p->vocab) > 8) return OT_ERR_UNSUPPORTED;
    if (check_strides) {
        if (p->stride_row < p->vocab || p->stride_depth < 0 || p->stride_seq < 0) return OT_ERR_INVALID_ARG;
    }
    return OT_OK;
}

BuildWorkspace carve_build_workspace(const ot_build_params& p, void* base) {
    const Frontier f = make_frontier(p.k, p.n, p.depth);
    const size_t rows = (size_t)p.batch * (size_t)(f.rows > p.n ? f.rows : p.n);
    const size_t parts = (size_t)scan_parts(p.vocab);
    const size_t k = (size_t)p.k;
    const size_t pool = (size_t)p.batch * p.depth * p.n;
    BuildWorkspace w;
    memset(&w, 0, sizeof(w));
    size_t off = 0;
    char* b = (char*)base;
    // (a null base is the sizing pass: offsets only)
    auto take = [&](size_t bytes) { char* q = b ? b + off : nullptr; off = align_up(off + bytes, 256); return (void*)q; };
    w.row_lse = (double*)take(rows * 8);
    w.row_topv = (float*)take(rows * k * 4);
    w.row_topi = (int32_t*)take(rows * k * 4);
    if (parts > 1) {
        w.part_m = (float*)take(rows * parts * 4);
        w.part_s = (double*)take(rows * parts * 8);
        w.part_topv = (float*)take(rows * parts * k * 4);
        w.part_topi = (int32_t*)take(rows * parts * k * 4);
    }
    w.pool_key = (double*)take(pool * 8);
    w.step_tau = (double*)take((size_t)p.batch * p.depth * 8);
    w.pool_tok = (int32_t*)take(pool * 4);
    w.pool_par = (int32_t*)take(pool * 4);
    w.pool_p = (double*)take(pool * 8);
    w.seq_E = (double*)take((size_t)p.batch * 8);
    w.seq_steps = (int32_t*)take((size_t)p.batch * 4);
    w.seq_active = (int32_t*)take((size_t)p.batch * 4);
    w.front_anc = (unsigned short*)take((size_t)2 * p.batch * p.n * OT_MAX_DEPTH * sizeof(unsigned short));
    w.bytes = off;
    return w;
}

static int check_tree_out(const ot_tree_out* o) {
    if (!o || !o->token || !o->parent || !o->depth || !o->score || !o->mask || !o->n_out || !o->expect)
        return OT_ERR_INVALID_ARG;
    if (((uintptr_t)o->mask % 8) || ((uintptr_t)o->expect % 8)) return OT_ERR_INVALID_ARG;
    return OT_OK;
}

__global__ void copy_i32_kernel(const int32_t* src, int32_t* dst, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = src[i];
}

static SelectGeometry select_geometry(const ot_build_params& p, const Frontier& f) {
    SelectGeometry g;
    g.batch = p.batch; g.k = p.k; g.n = p.n; g.depth = p.depth;
    g.rows_per_seq = f.rows;
    for (int i = 0; i < OT_MAX_DEPTH + 2; ++i) { g.F[i] = f.F[i]; g.row_start[i] = f.row_start[i]; }
    return g;
}

}  // namespace ot

using namespace ot;

extern "C" {

int ot_version(void) { return 100; }

const char* ot_status_string(int status) {
    switch (status) {
        case OT_OK: return "ok";
        case OT_ERR_INVALID_ARG: return "invalid argument";
        case OT_ERR_UNSUPPORTED: return "unsupported size or type";
        case OT_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case OT_ERR_HIP: return "HIP runtime error";
        case OT_ERR_SCRATCH_LIMIT: return "needs more scratch memory than the no-allocation entry point owns";
        default: return "unknown status";
    }
}

int ot_last_hip_error(void) { return g_last_hip_error; }

size_t ot_build_workspace_bytes(const ot_build_params* p) {
    if (validate_build(p, false) != OT_OK) return 0;
    return carve_build_workspace(*p, nullptr).bytes;
}

static int build_entry(const ot_build_params* p, const void* logits, void* workspace, size_t workspace_bytes,
                       const ot_tree_out* out, void* hip_stream, void* ev0, void* ev1) {
    int st = validate_build(p, true);
    if (st != OT_OK) return st;
    if (!logits || !workspace) return OT_ERR_INVALID_ARG;
    if ((uintptr_t)workspace % 16) return OT_ERR_INVALID_ARG;
    const int esize = p->logits_dtype == OT_BF16 ? 2 : 4;
    if ((uintptr_t)logits % esize) return OT_ERR_INVALID_ARG;
    st = check_tree_out(out);
    if (st != OT_OK) return st;
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    const Frontier f = make_frontier(p->k, p->n, p->depth);
    hipStream_t s = (hipStream_t)hip_stream;

    ScanGeometry sg;
    sg.batch = p->batch; sg.vocab = p->vocab; sg.k = p->k; sg.dtype = p->logits_dtype;
    sg.nsteps = p->depth; sg.rows_per_seq = f.rows;
    sg.grow_k = p->k; sg.grow_n = p->n;
    sg.stride_seq = p->stride_seq; sg.stride_depth = p->stride_depth; sg.stride_row = p->stride_row;
    st = launch_row_scan(sg, logits, ws, s, (hipEvent_t)ev0, (hipEvent_t)ev1);
    if (st != OT_OK) return st;
    return launch_tree_oneshot(select_geometry(*p, f), ws, *out, s);
}

int ot_build_tree(const ot_build_params* p, const void* logits, void* workspace, size_t workspace_bytes,
                  const ot_tree_out* out, void* hip_stream) {
    return build_entry(p, logits, workspace, workspace_bytes, out, hip_stream, nullptr, nullptr);
}

int ot_build_tree_timed(const ot_build_params* p, const void* logits, void* workspace, size_t workspace_bytes,
                        const ot_tree_out* out, void* hip_stream, void* scan_begin_event, void* scan_end_event) {
    return build_entry(p, logits, workspace, workspace_bytes, out, hip_stream, scan_begin_event, scan_end_event);
}

int ot_build_tree_adaptive(const ot_build_params* p, double delta, const void* logits, void* workspace,
                           size_t workspace_bytes, const ot_tree_out* out, int32_t* steps_used, double* e_sub,
                           void* hip_stream) {
    int st = validate_build(p, true);
    if (st != OT_OK) return st;
    if (!(delta == delta)) return OT_ERR_INVALID_ARG;
    if (!logits || !workspace || !steps_used || !e_sub) return OT_ERR_INVALID_ARG;
    if ((uintptr_t)workspace % 16 || (uintptr_t)steps_used % 4 || (uintptr_t)e_sub % 8) return OT_ERR_INVALID_ARG;
    const int esize = p->logits_dtype == OT_BF16 ? 2 : 4;
    if ((uintptr_t)logits % esize) return OT_ERR_INVALID_ARG;
    st = check_tree_out(out);
    if (st != OT_OK) return st;
    const Frontier f = make_frontier(p->k, p->n, p->depth);
    const SelectGeometry g = select_geometry(*p, f);
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = (hipStream_t)hip_stream;
    if (!tree_adaptive_supported(g)) {
        // Shapes beyond the single-wavefront kernel (n > 64, large pools): the loop of Algorithm 1 as the streaming
        // entry points run it, step by step on the stream -- scan of the step's F_t rows, selection, E_sub and the
        // loop condition, all decided on the device (a sequence that stops is frozen there: later steps skip it,
        // the final selection uses the layers it had), so the host neither waits nor reads anything back.  The
        // frontier lists and the per-step decisions land in the output arrays, which the final selection overwrites.
        st = launch_tree_begin(g, ws, s);
        if (st != OT_OK) return st;
        for (int t = 0; t < p->depth; ++t) {
            ScanGeometry sg;
            sg.batch = p->batch; sg.vocab = p->vocab; sg.k = p->k; sg.dtype = p->logits_dtype;
            sg.nsteps = 1; sg.rows_per_seq = f.F[t];
            sg.grow_k = 1; sg.grow_n = 1;
            sg.stride_seq = p->stride_seq; sg.stride_depth = 0; sg.stride_row = p->stride_row;
            st = launch_row_scan(sg, (const char*)logits + (size_t)t * p->stride_depth * esize, ws, s, nullptr, nullptr, true);
            if (st != OT_OK) return st;
            SelectGeometry gs = g;
            gs.rows_per_seq = f.F[t];
            st = launch_tree_step(gs, t, ws, out->token, out->parent, nullptr, s);
            if (st != OT_OK) return st;
            st = launch_tree_esub(g, t + 1, delta, ws, e_sub, out->depth, s);
            if (st != OT_OK) return st;
        }
        st = launch_tree_finalize(g, p->depth, ws, *out, s);
        if (st != OT_OK) return st;
        hipLaunchKernelGGL(copy_i32_kernel, dim3((p->batch + 255) / 256), dim3(256), 0, s, ws.seq_steps, steps_used, p->batch);
        OT_HIP_CHECK(hipGetLastError());
        return OT_OK;
    }
    ScanGeometry sg;
    sg.batch = p->batch; sg.vocab = p->vocab; sg.k = p->k; sg.dtype = p->logits_dtype;
    sg.nsteps = p->depth; sg.rows_per_seq = f.rows;
    sg.grow_k = p->k; sg.grow_n = p->n;
    sg.stride_seq = p->stride_seq; sg.stride_depth = p->stride_depth; sg.stride_row = p->stride_row;
    st = launch_row_scan(sg, logits, ws, s);
    if (st != OT_OK) return st;
    return launch_tree_adaptive(g, delta, ws, *out, steps_used, e_sub, s);
}

int ot_tree_begin(const ot_build_params* p, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int st = validate_build(p, false);
    if (st != OT_OK) return st;
    if (!workspace || (uintptr_t)workspace % 16) return OT_ERR_INVALID_ARG;
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    // every step overwrites the pool state it owns; only the per-sequence loop state (E = 0, no layer, not
    // stopped) has to be set
    return launch_tree_begin(select_geometry(*p, make_frontier(p->k, p->n, p->depth)), ws, (hipStream_t)hip_stream);
}

int ot_tree_expand(const ot_build_params* p, int32_t step, const void* rows, int64_t stride_seq, int64_t stride_row,
                   void* workspace, size_t workspace_bytes, int32_t* frontier_token, int32_t* frontier_parent_slot,
                   int32_t* frontier_count, void* hip_stream) {
    int st = validate_build(p, false);
    if (st != OT_OK) return st;
    if (step < 0 || step >= p->depth) return OT_ERR_INVALID_ARG;
    if (!rows || !workspace || !frontier_token || !frontier_parent_slot) return OT_ERR_INVALID_ARG;
    if ((uintptr_t)workspace % 16) return OT_ERR_INVALID_ARG;
    if (((uintptr_t)frontier_token % 4) || ((uintptr_t)frontier_parent_slot % 4) || ((uintptr_t)frontier_count % 4))
        return OT_ERR_INVALID_ARG;
    const int esize = p->logits_dtype == OT_BF16 ? 2 : 4;
    if ((uintptr_t)rows % esize) return OT_ERR_INVALID_ARG;
    if (stride_row < p->vocab || stride_seq < 0) return OT_ERR_INVALID_ARG;
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    const Frontier f = make_frontier(p->k, p->n, p->depth);
    hipStream_t s = (hipStream_t)hip_stream;

    ScanGeometry sg;
    sg.batch = p->batch; sg.vocab = p->vocab; sg.k = p->k; sg.dtype = p->logits_dtype;
    sg.nsteps = 1; sg.rows_per_seq = f.F[step];
    sg.grow_k = 1; sg.grow_n = 1;
    sg.stride_seq = stride_seq; sg.stride_depth = 0; sg.stride_row = stride_row;
    st = launch_row_scan(sg, rows, ws, s, nullptr, nullptr, true);      // rows of frozen sequences are not read
    if (st != OT_OK) return st;
    SelectGeometry g = select_geometry(*p, f);
    g.rows_per_seq = f.F[step];
    return launch_tree_step(g, step, ws, frontier_token, frontier_parent_slot, frontier_count, s);
}

int ot_tree_finalize(const ot_build_params* p, int32_t steps_done, void* workspace, size_t workspace_bytes,
                     const ot_tree_out* out, void* hip_stream) {
    int st = validate_build(p, false);
    if (st != OT_OK) return st;
    if (steps_done < 1 || steps_done > p->depth) return OT_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 16) return OT_ERR_INVALID_ARG;
    st = check_tree_out(out);
    if (st != OT_OK) return st;
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    const Frontier f = make_frontier(p->k, p->n, p->depth);
    return launch_tree_finalize(select_geometry(*p, f), steps_done, ws, *out, (hipStream_t)hip_stream);
}

int ot_tree_frontier_mask(const ot_build_params* p, int32_t steps_done, void* workspace, size_t workspace_bytes,
                          uint64_t* mask, void* hip_stream) {
    int st = validate_build(p, false);
    if (st != OT_OK) return st;
    if (steps_done < 1 || steps_done > p->depth) return OT_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 16 || !mask || (uintptr_t)mask % 8) return OT_ERR_INVALID_ARG;
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    const Frontier f = make_frontier(p->k, p->n, p->depth);
    return launch_tree_front_mask(select_geometry(*p, f), steps_done, ws, mask, OT_MASK_WORDS(p->depth * p->n),
                                  (hipStream_t)hip_stream);
}

int ot_tree_esub(const ot_build_params* p, int32_t steps_done, double delta, void* workspace, size_t workspace_bytes,
                 double* e_sub, int32_t* go_on, void* hip_stream) {
    int st = validate_build(p, false);
    if (st != OT_OK) return st;
    if (steps_done < 1 || steps_done > p->depth) return OT_ERR_INVALID_ARG;
    if (!(delta == delta)) return OT_ERR_INVALID_ARG;
    if (!workspace || (uintptr_t)workspace % 16 || !e_sub || !go_on) return OT_ERR_INVALID_ARG;
    if ((uintptr_t)e_sub % 8 || (uintptr_t)go_on % 4) return OT_ERR_INVALID_ARG;
    const BuildWorkspace ws = carve_build_workspace(*p, workspace);
    if (workspace_bytes < ws.bytes) return OT_ERR_WORKSPACE_TOO_SMALL;
    const Frontier f = make_frontier(p->k, p->n, p->depth);
    return launch_tree_esub(select_geometry(*p, f), steps_done, delta, ws, e_sub, go_on, (hipStream_t)hip_stream);
}

}  // extern "C"
