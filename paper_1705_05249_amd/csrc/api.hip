// Host-side boundary: argument validation, canonicalisation to the column-major form,
// configuration selection / override, and launch.  No allocation, no synchronisation, no
// host<->device copies happen here (paper Section 3.1: device pointers in, transfers left
// to the caller).  Validation touches no HIP API, so every error path can be exercised on
// a machine without a GPU.
#include <atomic>
#include <mutex>
#include <string>

#include "internal.h"
#include "select.h"
#include "lds_layout.h"

namespace mg {
namespace {

std::vector<KernelEntry> g_table;
std::once_flag g_once;

// Override state: set by the tuning calls, read by every GEMM call; relaxed atomics, so that a call racing with an
// override sees either the old or the new value of each word (kernel and split are checked together by legal()).
std::atomic<int32_t> g_override_kernel[2] = {{-1}, {-1}};   // per dtype
std::atomic<int32_t> g_override_split[2] = {{1}, {1}};
std::atomic<int32_t> g_override_batched{-1};
std::atomic<int32_t> g_fringe_mode{MG_FRINGE_AUTO};

const std::vector<KernelEntry> &table()
{
    std::call_once(g_once, [] {
        register_direct(g_table);
        register_mfma(g_table);
        register_gemv(g_table);
        register_batched(g_table);
        for (size_t i = 0; i < g_table.size(); ++i) g_table[i].cfg.kernel_id = static_cast<int32_t>(i);
    });
    return g_table;
}

bool valid_trans(int t) { return t == MG_NO_TRANS || t == MG_TRANS || t == MG_CONJ_TRANS; }

// Checks everything that does not need the pointers, in status-code order.
mg_status check_shape(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, int64_t lda, int64_t ldb,
                      int64_t ldc)
{
    if (layout != MG_ROW_MAJOR && layout != MG_COL_MAJOR) return MG_ERR_LAYOUT;
    if (!valid_trans(ta)) return MG_ERR_TRANS_A;
    if (!valid_trans(tb)) return MG_ERR_TRANS_B;
    if (m < 0 || n < 0 || k < 0) return MG_ERR_DIM;
    const int64_t lim = int64_t(1) << 31;          // each extent and each matrix must stay indexable
    if (m >= lim || n >= lim || k >= lim) return MG_ERR_DIM;
    const bool col = layout == MG_COL_MAJOR;
    const bool at = ta != MG_NO_TRANS, bt = tb != MG_NO_TRANS;
    // leading extent of each stored matrix
    const int64_t a_lead = col ? (at ? k : m) : (at ? m : k);
    const int64_t b_lead = col ? (bt ? n : k) : (bt ? k : n);
    const int64_t c_lead = col ? m : n;
    if (lda < (a_lead > 1 ? a_lead : 1)) return MG_ERR_LDA;
    if (ldb < (b_lead > 1 ? b_lead : 1)) return MG_ERR_LDB;
    if (ldc < (c_lead > 1 ? c_lead : 1)) return MG_ERR_LDC;
    const int64_t a_other = col ? (at ? m : k) : (at ? k : m);
    const int64_t b_other = col ? (bt ? k : n) : (bt ? n : k);
    const int64_t c_other = col ? n : m;
    const __int128 cap = __int128(1) << 40;        // elements; far beyond 288 GB, guards overflow
    if (__int128(lda) * a_other > cap || __int128(ldb) * b_other > cap || __int128(ldc) * c_other > cap)
        return MG_ERR_DIM;
    return MG_OK;
}

// Row-major C = op(A) op(B) is column-major C^T = op(B)^T op(A)^T on the same bytes:
// swap the operands and the roles of m and n.
Problem canonical(int dtype, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha,
                  const void *A, int64_t lda, const void *B, int64_t ldb, float beta, void *C, int64_t ldc,
                  void *ws, size_t ws_bytes, void *stream, int shape = MG_SHAPE_GENERAL)
{
    Problem p{};
    p.shape = shape;           // already in canonical terms: the caller knows the layout
    p.dtype = dtype;
    p.k = k;
    p.alpha = alpha;
    p.beta = beta;
    p.C = C;
    p.ldc = ldc;
    p.workspace = ws;
    p.workspace_bytes = ws_bytes;
    p.stream = static_cast<hipStream_t>(stream);
    const bool at = ta != MG_NO_TRANS, bt = tb != MG_NO_TRANS;
    if (layout == MG_COL_MAJOR) {
        p.m = m; p.n = n;
        p.A = A; p.lda = lda; p.a_trans = at;
        p.B = B; p.ldb = ldb; p.b_trans = bt;
    } else {
        p.m = n; p.n = m;
        p.A = B; p.lda = ldb; p.a_trans = bt;
        p.B = A; p.ldb = lda; p.b_trans = at;
    }
    return p;
}

int64_t problem_alignment(const Problem &p)
{
    int64_t a = pointer_alignment(p.A), b = pointer_alignment(p.B), c = pointer_alignment(p.C);
    int64_t r = a < b ? a : b;
    return r < c ? r : c;
}

// Picks the configuration for a canonical problem: the override if one is active, else the
// heuristic table.  Returns MG_OK and fills kernel/split, or an error.
// Fringe rows / columns of a ragged FP32 problem (fringe.h): a dimension that is 1 to 4 more than a multiple of
// the smallest tile.  Automatic mode takes them off where that saves at least ~1.5 % of the tiles and the sum is long
// enough for the problem to be bound by the matrix pipes rather than by memory (the fringe reads the other operand
// once more).  Measured on (4097, 129, 4095) with both operands along k: 67 -> 47 us.
void plan_fringe(Problem &p, bool forced)
{
    p.fringe_m = p.fringe_n = 0;
    const int mode = g_fringe_mode;
    if (mode == MG_FRINGE_OFF || (forced && mode != MG_FRINGE_ON)) return;
    if (p.dtype != MG_F32 || p.shape != MG_SHAPE_GENERAL || p.mask_c || p.conv != nullptr || p.alpha == 0.f || p.k == 0) return;
    if (p.m < 64 || p.n < 64) return;
    if (mode == MG_FRINGE_AUTO && p.k < 256) return;
    auto extra = [&](int64_t d) {
        const int64_t r = d % 64;
        return r >= 1 && r <= 4 && (mode == MG_FRINGE_ON || d <= 4160) ? static_cast<int>(r) : 0;
    };
    p.fringe_m = extra(p.m);
    p.fringe_n = extra(p.n);
}

// Also decides the problem's fringe (p.fringe_m, p.fringe_n).
mg_status choose(Problem &p, int64_t alignment, size_t workspace_bytes, int32_t *kernel, int32_t *split)
{
    const auto &t = table();
    const int32_t forced = g_override_kernel[p.dtype];
    plan_fringe(p, forced >= 0);
    if (forced >= 0) {
        const KernelEntry &e = t[forced];
        const int32_t forced_split = g_override_split[p.dtype];
        if (!e.legal || !e.legal(p, forced_split, alignment)) return MG_ERR_CONFIG;
        *kernel = forced;
        *split = forced_split;
        return MG_OK;
    }
    select_config(t, p, alignment, workspace_bytes, kernel, split);
    if (*kernel < 0 && (p.fringe_m != 0 || p.fringe_n != 0)) {
        p.fringe_m = p.fringe_n = 0;                   // no kernel for the problem less its fringe: the whole problem
        select_config(t, p, alignment, workspace_bytes, kernel, split);
    }
    if (*kernel < 0) return MG_ERR_CONFIG;
    return MG_OK;
}

size_t round_up_256(size_t v) { return (v + 255) / 256 * 256; }

// Indirect GEMM, the paper's Section 3.2 route for problems that break the fast kernel's assumptions: copy the
// operands into zero-padded, aligned buffers whose sizes are whole tiles, run the fast kernel there, copy the
// result back.  FP16 needs it most: ragged or unaligned FP16 problems otherwise run the bounds-checked
// register-staged kernels at 0.2-0.6 of the direct-to-LDS rate (4097^3: 525 us; an odd leading dimension puts
// every other row at 2-byte alignment), while the copies are O(n^2) (~30 us at 4097^3).  FP32 loses ~20 % in
// its bounds-checked flavour plus what ragged sizes lose to tile quantisation: large problems gain.  The padded buffers live in
// the caller's workspace; without enough of it the direct route runs.  One rounding as always: the fast
// kernel applies alpha and beta in the padded C, whose leading part is then copied out bit for bit.
struct IndirectPlan {
    int64_t mp, np, kp;
    size_t a_bytes, b_bytes, c_bytes;
    size_t total() const { return a_bytes + b_bytes + c_bytes; }
};

bool indirect_plan(const Problem &p, bool pointers_known, IndirectPlan *plan)
{
    if (p.shape != MG_SHAPE_GENERAL || p.alpha == 0.f || p.k == 0) return false;
    if (g_override_kernel[p.dtype] >= 0) return false;                 // a forced kernel gets the problem as it is
    const double work = static_cast<double>(p.m) * static_cast<double>(p.n) * static_cast<double>(p.k);
    const size_t elem = p.elem();
    int64_t tile = 0, ktile = 0;
    if (p.dtype == MG_F16) {
        // four extra launches and ~33 us of copies at 4096^2: measured a loss at 1000^3 (28 against 22 us), a gain
        // at 2049^3 (56 against 96 us)
        if (p.m < 1024 || p.n < 1024 || p.k < 256 || work < 2.0e9) return false;
        const bool whole = p.m % 128 == 0 && p.n % 128 == 0 && p.k % 64 == 0;
        const bool aligned = p.lda % 8 == 0 && p.ldb % 8 == 0 &&
                             (!pointers_known || (pointer_alignment(p.A) >= 16 && pointer_alignment(p.B) >= 16));
        if (whole && aligned) return false;                            // the fast kernels take it directly
        // Operands whose rows start on dwords run most of their K-tiles on the fast flavour's schedule inside the
        // bounds-checked kernels, and the copies pay only where the product is long next to the matrices: below about
        // 900 multiply-adds per element moved the direct route wins (re-measured with the copies of C gone from the
        // larger problems, direct / through the copies: 2051^3 42-44 / 47, 2501^3 56 / 57, 2801^3 66-68 / 69-71, 3001^3
        // 73-86 / 71-73, (2051, 2051, 8201) 142-161 / 126-127).  Even leading dimensions, us direct / through
        // the copies (A along m | along k): 1300^3 17.6 / 25.0 | 15.6 / 23.5, 1800^3 25.9 / 32.6 | 24.7 / 30.8, 2050^3
        // 46.5 / 46.4 | 46.2 / 45.8, 2500^3 62.2 / 55.4 | 55.5 / 55.3, 3000^3 81.7 / 74.7 | 65.4 / 74.2, 3500^3 115 / 98 |
        // 96 / 97, 4104^3 205 / 196, 6002^3 533 / 442 | 572 / 441; (4100, 4100, 512) 43.7 / 52.0 | 36.5 / 50.0,
        // (8200, 1030, 2050) 60.9 / 78.1 | 53.9 / 81.5, (2050, 2050, 8200) 126 / 126 | 120 / 123.  (Without the
        // pointers, for the workspace query, the copies are assumed: an upper bound.)
        const bool dword_rows = p.lda % 2 == 0 && p.ldb % 2 == 0 && pointers_known && pointer_alignment(p.A) >= 4 &&
                                pointer_alignment(p.B) >= 4;
        const double moved = static_cast<double>(p.m) * p.k + static_cast<double>(p.k) * p.n + static_cast<double>(p.m) * p.n;
        if (dword_rows && work < 900.0 * moved) return false;
        tile = p.m >= 2048 && p.n >= 2048 ? 256 : 128;
        ktile = 64;
    } else {
        // FP32 does not take this route.  It did while the bounds-checked flavour ran at ~0.78 of the whole-tile rate
        // (4000^3: 1150 us direct, 978 us through the copies); since that flavour runs its whole K-tiles on the fast
        // flavour's schedule, partial tiles included, the direct route wins: 2049^3 195 / 138 us (A along m / k)
        // against 200, 3000^3 430 / 417 against 473, 4000^3 927 / 896 against 977, 4097^3 1020 / 945 against 1139,
        // 5001^3 1990 / 1940 against 2068 (the copies cost ~70 us at 4096^2).
        return false;
    }
    plan->mp = ceil_div(p.m, tile) * tile;
    plan->np = ceil_div(p.n, tile) * tile;
    plan->kp = ceil_div(p.k, ktile) * ktile;
    plan->a_bytes = round_up_256(static_cast<size_t>(plan->mp) * plan->kp * elem);
    plan->b_bytes = round_up_256(static_cast<size_t>(plan->kp) * plan->np * elem);
    plan->c_bytes = round_up_256(static_cast<size_t>(plan->mp) * plan->np * elem);
    return true;
}

mg_status run_canonical(Problem p);

mg_status run_indirect(const Problem &p, const IndirectPlan &plan)
{
    char *ws = static_cast<char *>(p.workspace);
    void *ap = ws, *bp = ws + plan.a_bytes, *cp = ws + plan.a_bytes + plan.b_bytes;
    hipStream_t st = p.stream;
    // an operand keeps its storage order: stored rows x columns (column-major view) = m x k or k x m
    const int64_t a_minor = p.a_trans ? p.k : p.m, a_major = p.a_trans ? p.m : p.k;
    const int64_t a_minor_p = p.a_trans ? plan.kp : plan.mp, a_major_p = p.a_trans ? plan.mp : plan.kp;
    const int64_t b_minor = p.b_trans ? p.n : p.k, b_major = p.b_trans ? p.k : p.n;
    const int64_t b_minor_p = p.b_trans ? plan.np : plan.kp, b_major_p = p.b_trans ? plan.kp : plan.np;
    const PadCopy copies[3] = {{a_minor, a_major, p.A, p.lda, ap, a_minor_p, a_minor_p, a_major_p},
                               {b_minor, b_major, p.B, p.ldb, bp, b_minor_p, b_minor_p, b_major_p},
                               {p.m, p.n, p.C, p.ldc, cp, plan.mp, plan.mp, plan.np}};
    Problem q = p;
    q.m = plan.mp; q.n = plan.np; q.k = plan.kp;
    q.A = ap; q.lda = a_minor_p;
    q.B = bp; q.ldb = b_minor_p;
    {
        // Where a kernel with direct-to-LDS loads and a bounds-checked epilogue takes the padded product, only A and B
        // are copied and C stays where it is: no copy of C in (beta != 0) and none out (each ~12 us at 4097^2 FP16, plus
        // the 3.5-4 us gap of a dependent launch).
        Problem direct_c = q;
        direct_c.clip_m = p.m;
        direct_c.clip_n = p.n;
        direct_c.workspace = nullptr;
        direct_c.workspace_bytes = 0;
        // (only where the padded product would run on a tile that has such a flavour anyway: forced onto the 256 x 256
        // tile, 2051^3, which prefers smaller ones, took 53.7 us against 46 us with the copies)
        Problem padded = q;
        padded.C = cp;
        padded.ldc = plan.mp;
        int32_t wanted = -1, wanted_split = 1, kernel = -1, split = 1;
        const bool unsplit = choose(padded, problem_alignment(padded), 0, &wanted, &wanted_split) == MG_OK && wanted_split == 1;
        if (unsplit && choose(direct_c, problem_alignment(direct_c), 0, &kernel, &split) == MG_OK && split == 1 &&
            table()[kernel].cfg.tile_m == table()[wanted].cfg.tile_m && table()[kernel].cfg.tile_n == table()[wanted].cfg.tile_n &&
            table()[kernel].cfg.waves_m * table()[kernel].cfg.waves_n == table()[wanted].cfg.waves_m * table()[wanted].cfg.waves_n) {
            if (launch_pad_matrices(p.dtype, copies, 2, st) != hipSuccess) return MG_ERR_LAUNCH;
            return table()[kernel].launch(direct_c, 1) == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
        }
    }
    if (launch_pad_matrices(p.dtype, copies, p.beta != 0.f ? 3 : 2, st) != hipSuccess) return MG_ERR_LAUNCH;
    q.C = cp; q.ldc = plan.mp;
    const size_t used = plan.total();
    q.workspace = p.workspace_bytes > used ? ws + used : nullptr;
    q.workspace_bytes = p.workspace_bytes > used ? p.workspace_bytes - used : 0;
    const mg_status s = run_canonical(q);
    if (s != MG_OK) return s;
    return launch_unpad_matrix(p.dtype, p.m, p.n, cp, plan.mp, p.C, p.ldc, st) == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

// Selects and launches the configuration for a canonical problem with at least one output.
mg_status run_canonical(Problem p)
{
    IndirectPlan plan;
    // (the copy back out of the padded result writes all of C: not for a call that may only touch a triangle)
    if (!p.mask_c && indirect_plan(p, true, &plan) && p.workspace != nullptr && pointer_alignment(p.workspace) >= 256 &&
        p.workspace_bytes >= plan.total())
        return run_indirect(p, plan);
    int32_t kernel = -1, split = 1;
    const bool ws_usable = p.workspace != nullptr && pointer_alignment(p.workspace) >= 256;
    const mg_status s = choose(p, problem_alignment(p), ws_usable ? p.workspace_bytes : 0, &kernel, &split);
    if (s != MG_OK) return s;
    const KernelEntry &e = table()[kernel];
    if (p.mask_c && !e.masks_triangle) return MG_ERR_CONFIG;      // the caller takes the route that sets the rest of C aside
    const size_t need = e.workspace(p, split);
    if (need > 0 && !(ws_usable && p.workspace_bytes >= need)) return MG_ERR_WORKSPACE;
    return e.launch(p, split) == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

// shape: a ProblemShape hint in terms of the canonical (column-major) problem, see canonical()
mg_status run_gemm(int dtype, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha,
                   const void *A, int64_t lda, const void *B, int64_t ldb, float beta, void *C, int64_t ldc,
                   void *ws, size_t ws_bytes, void *stream, int shape = MG_SHAPE_GENERAL)
{
    mg_status s = check_shape(layout, ta, tb, m, n, k, lda, ldb, ldc);
    if (s != MG_OK) return s;
    if (m == 0 || n == 0) return MG_OK;
    const bool reads_ab = alpha != 0.f && k != 0;
    if (C == nullptr || (reads_ab && (A == nullptr || B == nullptr))) return MG_ERR_NULL;
    Problem p = canonical(dtype, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, ws, ws_bytes, stream, shape);
    return run_canonical(p);
}

// Matrix-vector product as the one-row canonical problem  y^T = x^T op(A)^T: x is the 1 x K operand
// with leading dimension incx, op(A)^T the K x M operand read in place, y the 1 x M result with leading
// dimension incy.  The matrix-vector kernels take all three strides as they are.
mg_status check_gemv(int layout, int trans, int64_t m, int64_t n, int64_t lda, int64_t incx, int64_t incy)
{
    if (layout != MG_ROW_MAJOR && layout != MG_COL_MAJOR) return MG_ERR_LAYOUT;
    if (!valid_trans(trans)) return MG_ERR_TRANS_A;
    const int64_t lim = int64_t(1) << 31;
    if (m < 0 || n < 0 || m >= lim || n >= lim) return MG_ERR_DIM;
    const int64_t lead = layout == MG_COL_MAJOR ? m : n;
    if (lda < (lead > 1 ? lead : 1)) return MG_ERR_LDA;
    if (incx < 1 || incy < 1 || incx >= lim || incy >= lim) return MG_ERR_INC;
    // the same cap as for GEMM operands: the matrix and both strided vectors stay far below 2^63 bytes
    const int64_t other = layout == MG_COL_MAJOR ? n : m;
    const __int128 cap = __int128(1) << 40;
    if (__int128(lda) * other > cap || __int128(incx) * (m > n ? m : n) > cap || __int128(incy) * (m > n ? m : n) > cap)
        return MG_ERR_DIM;
    return MG_OK;
}

Problem gemv_problem(int dtype, int layout, int trans, int64_t m, int64_t n, float alpha, const void *A, int64_t lda,
                     const void *x, int64_t incx, float beta, void *y, int64_t incy, void *ws, size_t ws_bytes,
                     void *stream)
{
    const bool t = trans != MG_NO_TRANS;
    Problem p{};
    p.dtype = dtype;
    p.m = 1; p.n = t ? n : m; p.k = t ? m : n;
    p.A = x; p.lda = incx; p.a_trans = false;
    // op(A)^T (l, j) = op(A)(j, l): contiguous along the outputs exactly when the stored matrix has its
    // unit stride along op(A)'s rows
    p.B = A; p.ldb = lda; p.b_trans = (layout == MG_COL_MAJOR) != t;
    p.C = y; p.ldc = incy;
    p.alpha = alpha; p.beta = beta;
    p.workspace = ws; p.workspace_bytes = ws_bytes;
    p.stream = static_cast<hipStream_t>(stream);
    return p;
}

mg_status run_gemv(int dtype, int layout, int trans, int64_t m, int64_t n, float alpha, const void *A, int64_t lda,
                   const void *x, int64_t incx, float beta, void *y, int64_t incy, void *ws, size_t ws_bytes,
                   void *stream)
{
    const mg_status s = check_gemv(layout, trans, m, n, lda, incx, incy);
    if (s != MG_OK) return s;
    Problem p = gemv_problem(dtype, layout, trans, m, n, alpha, A, lda, x, incx, beta, y, incy, ws, ws_bytes, stream);
    if (p.n == 0) return MG_OK;
    const bool reads = alpha != 0.f && p.k != 0;
    if (y == nullptr || (reads && (A == nullptr || x == nullptr))) return MG_ERR_NULL;
    return run_canonical(p);
}

// Canonicalises a (generic or strided) batched call to column-major and launches it.
mg_status run_batched(BatchedProblem &p, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                      const void *A, const int64_t *a_off, int64_t stride_a, int64_t lda, const void *B,
                      const int64_t *b_off, int64_t stride_b, int64_t ldb, void *C, const int64_t *c_off,
                      int64_t stride_c, int64_t ldc, int64_t batch, void *stream)
{
    const bool at = ta != MG_NO_TRANS, bt = tb != MG_NO_TRANS;
    p.k = k;
    p.C = C; p.c_off = c_off; p.stride_c = stride_c; p.ldc = ldc;
    p.batch = batch;
    p.stream = static_cast<hipStream_t>(stream);
    if (layout == MG_COL_MAJOR) {
        p.m = m; p.n = n;
        p.A = A; p.a_off = a_off; p.stride_a = stride_a; p.lda = lda; p.a_trans = at;
        p.B = B; p.b_off = b_off; p.stride_b = stride_b; p.ldb = ldb; p.b_trans = bt;
    } else {
        p.m = n; p.n = m;
        p.A = B; p.a_off = b_off; p.stride_a = stride_b; p.lda = ldb; p.a_trans = bt;
        p.B = A; p.b_off = a_off; p.stride_b = stride_a; p.ldb = lda; p.b_trans = at;
    }
    const auto &t = table();
    int32_t kernel = -1;
    const int32_t forced = g_override_batched;
    if (forced >= 0) {
        const KernelEntry &e = t[forced];
        if (!e.legal_batched || !e.legal_batched(p)) return MG_ERR_CONFIG;
        kernel = forced;
    } else {
        kernel = select_batched(t, p);
        if (kernel < 0) return MG_ERR_CONFIG;
    }
    return t[kernel].launch_batched(p) == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}


mg_status generic_batched(int dtype, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, const float *alphas,
                          const void *A, const int64_t *a_offsets, int64_t lda, const void *B,
                          const int64_t *b_offsets, int64_t ldb, const float *betas, void *C,
                          const int64_t *c_offsets, int64_t ldc, int64_t batch_count, void *stream)
{
    mg_status s = check_shape(layout, ta, tb, m, n, k, lda, ldb, ldc);
    if (s != MG_OK) return s;
    if (batch_count < 0 || batch_count >= (int64_t(1) << 31)) return MG_ERR_BATCH;
    if (m == 0 || n == 0 || batch_count == 0) return MG_OK;
    if (!alphas || !betas || !a_offsets || !b_offsets || !c_offsets || !C) return MG_ERR_NULL;
    if (k != 0 && (!A || !B)) return MG_ERR_NULL;
    BatchedProblem p{};
    p.dtype = dtype;
    p.alphas = alphas; p.betas = betas;
    return run_batched(p, layout, ta, tb, m, n, k, A, a_offsets, 0, lda, B, b_offsets, 0, ldb, C, c_offsets, 0, ldc,
                       batch_count, stream);
}

mg_status strided_batched(int dtype, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha,
                          const void *A, int64_t lda, int64_t stride_a, const void *B, int64_t ldb, int64_t stride_b,
                          float beta, void *C, int64_t ldc, int64_t stride_c, int64_t batch_count, void *stream)
{
    mg_status s = check_shape(layout, ta, tb, m, n, k, lda, ldb, ldc);
    if (s != MG_OK) return s;
    if (batch_count < 0 || batch_count >= (int64_t(1) << 31)) return MG_ERR_BATCH;
    if (stride_a < 0 || stride_b < 0 || stride_c < 0) return MG_ERR_STRIDE;
    if (m == 0 || n == 0 || batch_count == 0) return MG_OK;
    if (!C) return MG_ERR_NULL;
    if (k != 0 && alpha != 0.f && (!A || !B)) return MG_ERR_NULL;
    BatchedProblem p{};
    p.dtype = dtype;
    p.strided = true;
    p.alpha = alpha; p.beta = beta;
    return run_batched(p, layout, ta, tb, m, n, k, A, nullptr, stride_a, lda, B, nullptr, stride_b, ldb, C, nullptr,
                       stride_c, ldc, batch_count, stream);
}

// Checks a convolution geometry; fills the output extents and K = channels * kernel_h * kernel_w.
mg_status check_conv(const ConvShape &s, int64_t filters, int64_t *out_h, int64_t *out_w, int64_t *k)
{
    if (s.channels < 1 || s.height < 1 || s.width < 1 || s.kernel_h < 1 || s.kernel_w < 1 || s.pad_h < 0 ||
        s.pad_w < 0 || s.stride_h < 1 || s.stride_w < 1 || s.dilation_h < 1 || s.dilation_w < 1 || filters < 0)
        return MG_ERR_CONV;
    const int64_t lim = int64_t(1) << 31;
    if (s.channels >= lim || s.height >= lim || s.width >= lim || s.kernel_h >= lim || s.kernel_w >= lim ||
        s.pad_h >= lim || s.pad_w >= lim || s.stride_h >= lim || s.stride_w >= lim || s.dilation_h >= lim ||
        s.dilation_w >= lim || filters >= lim)
        return MG_ERR_DIM;
    *out_h = conv_out_extent(s.height, s.kernel_h, s.pad_h, s.stride_h, s.dilation_h);
    *out_w = conv_out_extent(s.width, s.kernel_w, s.pad_w, s.stride_w, s.dilation_w);
    // the unfold kernel indexes one image plane and the padded input window with 32-bit integers
    if (__int128(s.height) * s.width >= lim) return MG_ERR_DIM;
    if (s.height + 2 * s.pad_h >= lim || s.width + 2 * s.pad_w >= lim ||
        s.pad_h + __int128(s.dilation_h) * (s.kernel_h - 1) >= lim || s.pad_w + __int128(s.dilation_w) * (s.kernel_w - 1) >= lim)
        return MG_ERR_DIM;
    const __int128 kk = __int128(s.channels) * s.kernel_h * s.kernel_w;
    const __int128 total = kk * *out_h * *out_w;
    if (kk >= lim || total >= lim || __int128(s.channels) * s.height * s.width >= (__int128(1) << 40)) return MG_ERR_DIM;
    *k = static_cast<int64_t>(kk);
    return MG_OK;
}

// a 1x1 filter with unit stride and no padding: the column matrix is the image itself
bool conv_is_plain_gemm(const ConvShape &s)
{
    return s.kernel_h == 1 && s.kernel_w == 1 && s.pad_h == 0 && s.pad_w == 0 && s.stride_h == 1 && s.stride_w == 1;
}


mg_status run_im2col(int dtype, const ConvShape &s, const void *im, void *col, void *stream)
{
    int64_t out_h, out_w, k;
    mg_status st = check_conv(s, 0, &out_h, &out_w, &k);
    if (st != MG_OK) return st;
    if (out_h == 0 || out_w == 0) return MG_OK;
    if (im == nullptr || col == nullptr) return MG_ERR_NULL;
    return launch_im2col(dtype, s, im, col, static_cast<hipStream_t>(stream)) == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

// The convolution as one GEMM launch whose op(A) is gathered from the image (kernels of the family MG_FAMILY_CONV):
// the configuration is the one automatic selection gives the GEMM on a stored column matrix, if that is a kernel
// with such a variant (the 64 x 64 tile "mk" kernels, with their slices of the sum) and the layer is one where the
// gather pays, or the forced configuration if that is of the family.  MG_ERR_CONFIG: no such kernel, take the unfold route.
mg_status run_conv2d_fused(int dtype, const ConvShape &s, int64_t filters, int64_t n, int64_t k, float alpha, const void *im,
                           const void *weights, float beta, void *out, void *ws, size_t ws_bytes, void *stream)
{
    const auto &t = table();
    // canonical (column-major) form of the row-major product: m = output positions, n = filters
    Problem p = canonical(dtype, MG_ROW_MAJOR, MG_NO_TRANS, MG_NO_TRANS, filters, n, k, alpha, weights, k, nullptr, n, beta,
                          out, n, ws, ws_bytes, stream);
    int32_t kernel = -1, split = 1;
    const int32_t forced = g_override_kernel[dtype];
    if (forced >= 0) {
        if (t[forced].cfg.family != MG_FAMILY_CONV) return MG_ERR_CONFIG;       // a forced GEMM kernel: the unfold route
        kernel = forced;
        split = g_override_split[dtype];
    } else {
        // Measured on the four benchmark layers (FP16, us, fused / unfold route): 147 rows of the column matrix and 64
        // filters 9.4 / 12.2; 576 rows, 128 filters 16.9 / 14.0; 1152 rows, 256 filters 30 (15.5 in four slices) /
        // 14.9; 2304 rows, 512 filters 55 (20 in four slices) / 17.5.  A gathered K-tile takes about 1.5 us against
        // 1.0 us for a stored one (each element is a load of its own behind index arithmetic), and every tile column
        // of filters gathers the same elements again: the fused route pays where the sum is a few K-tiles and the
        // filters are one tile column.
        if (k > 256 || filters > 64) return MG_ERR_CONFIG;
        int32_t plain = -1;
        select_config(t, p, 256, ws_bytes, &plain, &split);
        if (plain < 0) return MG_ERR_CONFIG;
        const std::string name = t[plain].name;
        const char *fused = nullptr;
        if (name == "hmfma_64x64x64_w2x2_mk" || name == "hmfma_64x64x64_w2x2_mk_edge") fused = "hconv_64x64x64_w2x2";
        else if (name == "smfma_64x64x32_w2x2_mk" || name == "smfma_64x64x32_w2x2_mk_edge") fused = "sconv_64x64x32_w2x2";
        if (fused == nullptr) return MG_ERR_CONFIG;
        for (size_t i = 0; i < t.size(); ++i)
            if (std::string(t[i].name) == fused) kernel = static_cast<int32_t>(i);
        if (kernel < 0) return MG_ERR_CONFIG;
    }
    p.A = im;
    p.conv = &s;
    const KernelEntry &e = t[kernel];
    if (!e.legal || !e.legal(p, split, problem_alignment(p))) return MG_ERR_CONFIG;
    const size_t need = e.workspace ? e.workspace(p, split) : 0;
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return forced >= 0 ? MG_ERR_WORKSPACE : MG_ERR_CONFIG;
    return e.launch(p, split) == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

// out (filters x OH*OW) = alpha * weights (filters x K) * col (K x OH*OW) + beta * out, all row-major; the
// column matrix sits at the start of the workspace, the GEMM's own scratch (split-K) behind it
mg_status run_conv2d(int dtype, const ConvShape &s, int64_t filters, float alpha, const void *im, const void *weights,
                     float beta, void *out, void *ws, size_t ws_bytes, void *stream)
{
    int64_t out_h, out_w, k;
    mg_status st = check_conv(s, filters, &out_h, &out_w, &k);
    if (st != MG_OK) return st;
    const int64_t n = out_h * out_w;
    if (filters == 0 || n == 0) return MG_OK;
    if (out == nullptr || (alpha != 0.f && (im == nullptr || weights == nullptr))) return MG_ERR_NULL;
    const size_t elem = dtype == MG_F32 ? 4 : 2;
    const void *col = im;
    size_t col_bytes = 0;
    const bool plain = conv_is_plain_gemm(s);
    const int32_t forced = g_override_kernel[dtype];
    const bool forced_conv = forced >= 0 && table()[forced].cfg.family == MG_FAMILY_CONV;
    if (alpha != 0.f && (!plain || forced_conv)) {
        if (!plain) {
            col_bytes = round_up_256(static_cast<size_t>(k) * n * elem);
            if (ws == nullptr || pointer_alignment(ws) < 256 || ws_bytes < col_bytes) return MG_ERR_WORKSPACE;
        }
        // Without the unfold pass where a kernel that gathers op(A) from the image exists for the configuration the
        // GEMM would get: the caller's workspace then only serves the slices of the sum.
        mg_status fused = run_conv2d_fused(dtype, s, filters, n, k, alpha, im, weights, beta, out, ws, ws_bytes, stream);
        if (fused != MG_ERR_CONFIG || forced_conv) return fused;
        if (launch_im2col(dtype, s, im, ws, static_cast<hipStream_t>(stream)) != hipSuccess) return MG_ERR_LAUNCH;
        col = ws;
    }
    void *rest = ws == nullptr ? nullptr : static_cast<char *>(ws) + col_bytes;
    const size_t rest_bytes = ws_bytes > col_bytes ? ws_bytes - col_bytes : 0;
    return run_gemm(dtype, MG_ROW_MAJOR, MG_NO_TRANS, MG_NO_TRANS, filters, n, k, alpha, weights, k, col, n, beta, out,
                    n, rest_bytes ? rest : nullptr, rest_bytes, stream);
}

// ---- GEMM-derived level-3 routines: a support kernel makes the special operand general (or sets the
// untouched part of C aside), then the product is run_gemm.  Workspace layout: the dense operand(s) first,
// each rounded up to 256 bytes, the GEMM's own scratch (split-K) behind them.

bool valid_side(int v) { return v == MG_LEFT || v == MG_RIGHT; }
bool valid_uplo(int v) { return v == MG_UPPER || v == MG_LOWER; }
bool valid_diag(int v) { return v == MG_NON_UNIT || v == MG_UNIT; }

// the stored triangle as it appears in the column-major view of the bytes
bool lower_in_view(int layout, int uplo) { return (layout == MG_COL_MAJOR) == (uplo == MG_LOWER); }

struct Carve {
    char *at;
    size_t left;
    bool ok;
    Carve(void *ws, size_t bytes) : at(static_cast<char *>(ws)), left(bytes), ok(ws != nullptr && pointer_alignment(ws) >= 256) {}
    void *take(size_t bytes)
    {
        bytes = round_up_256(bytes);
        if (!ok || left < bytes) { ok = false; return nullptr; }
        void *p = at;
        at += bytes;
        left -= bytes;
        return p;
    }
    void *rest() const { return ok && left > 0 ? at : nullptr; }
};

mg_status check_symm(int layout, int side, int uplo, int64_t m, int64_t n, int64_t lda, int64_t ldb, int64_t ldc)
{
    if (layout != MG_ROW_MAJOR && layout != MG_COL_MAJOR) return MG_ERR_LAYOUT;
    if (!valid_side(side)) return MG_ERR_SIDE;
    if (!valid_uplo(uplo)) return MG_ERR_UPLO;
    const int64_t lim = int64_t(1) << 31;
    if (m < 0 || n < 0 || m >= lim || n >= lim) return MG_ERR_DIM;
    const int64_t ka = side == MG_LEFT ? m : n, lead = layout == MG_COL_MAJOR ? m : n;
    if (lda < (ka > 1 ? ka : 1)) return MG_ERR_LDA;
    if (ldb < (lead > 1 ? lead : 1)) return MG_ERR_LDB;
    if (ldc < (lead > 1 ? lead : 1)) return MG_ERR_LDC;
    if (ka > 64 * 65535) return MG_ERR_DIM;
    return MG_OK;
}

mg_status run_symm(int dtype, int layout, int side, int uplo, int64_t m, int64_t n, float alpha, const void *A, int64_t lda,
                   const void *B, int64_t ldb, float beta, void *C, int64_t ldc, void *ws, size_t ws_bytes, void *stream)
{
    const mg_status s = check_symm(layout, side, uplo, m, n, lda, ldb, ldc);
    if (s != MG_OK) return s;
    if (m == 0 || n == 0) return MG_OK;
    if (C == nullptr || (alpha != 0.f && (A == nullptr || B == nullptr))) return MG_ERR_NULL;
    if (alpha == 0.f) {     // C <- beta * C: an empty product (the unused leading dimensions only have to be legal)
        const int64_t any = m > n ? m : n;
        return run_gemm(dtype, layout, MG_NO_TRANS, MG_NO_TRANS, m, n, 0, 0.f, nullptr, any, nullptr, any, beta, C, ldc,
                        nullptr, 0, stream);
    }
    const int64_t ka = side == MG_LEFT ? m : n;
    const size_t elem = dtype == MG_F32 ? 4 : 2;
    Carve carve(ws, ws_bytes);
    void *full = carve.take(static_cast<size_t>(ka) * ka * elem);
    if (full == nullptr) return MG_ERR_WORKSPACE;
    if (launch_expand_symmetric(dtype, ka, A, lda, lower_in_view(layout, uplo), full, static_cast<hipStream_t>(stream)) !=
        hipSuccess)
        return MG_ERR_LAUNCH;
    // a symmetric dense matrix with leading dimension ka reads the same in either layout
    if (side == MG_LEFT)
        return run_gemm(dtype, layout, MG_NO_TRANS, MG_NO_TRANS, m, n, m, alpha, full, ka, B, ldb, beta, C, ldc, carve.rest(),
                        carve.left, stream);
    return run_gemm(dtype, layout, MG_NO_TRANS, MG_NO_TRANS, m, n, n, alpha, B, ldb, full, ka, beta, C, ldc, carve.rest(),
                    carve.left, stream);
}

mg_status check_syrk(int layout, int uplo, int trans, int64_t n, int64_t k, int64_t lda, int64_t ldc)
{
    if (layout != MG_ROW_MAJOR && layout != MG_COL_MAJOR) return MG_ERR_LAYOUT;
    if (!valid_uplo(uplo)) return MG_ERR_UPLO;
    if (!valid_trans(trans)) return MG_ERR_TRANS_A;
    const int64_t lim = int64_t(1) << 31;
    if (n < 0 || k < 0 || n >= lim || k >= lim) return MG_ERR_DIM;
    // A is n x k (no transpose) or k x n as stored
    const bool rows_are_n = trans == MG_NO_TRANS;
    const int64_t lead = (layout == MG_COL_MAJOR) == rows_are_n ? n : k;
    if (lda < (lead > 1 ? lead : 1)) return MG_ERR_LDA;
    if (ldc < (n > 1 ? n : 1)) return MG_ERR_LDC;
    return MG_OK;
}

mg_status run_syrk(int dtype, int layout, int uplo, int trans, int64_t n, int64_t k, float alpha, const void *A, int64_t lda,
                   float beta, void *C, int64_t ldc, void *ws, size_t ws_bytes, void *stream)
{
    const mg_status s = check_syrk(layout, uplo, trans, n, k, lda, ldc);
    if (s != MG_OK) return s;
    if (n == 0) return MG_OK;
    const bool reads_a = alpha != 0.f && k != 0;
    if (C == nullptr || (reads_a && A == nullptr)) return MG_ERR_NULL;
    const size_t elem = dtype == MG_F32 ? 4 : 2;
    const bool other_is_lower = !lower_in_view(layout, uplo);
    const bool nt0 = trans == MG_NO_TRANS;
    Carve carve(ws, ws_bytes);
    void *aside = carve.take(static_cast<size_t>(n) * n * elem);
    if (aside == nullptr) return MG_ERR_WORKSPACE;          // the contract is the same whichever route runs
    // First choice: one launch of a macro-tile kernel whose epilogue writes the referenced triangle only (tiles wholly
    // outside it are skipped, tiles on the diagonal store with a mask).  Not for problems the padded-copy route would
    // take, and not when the kernel in charge (small problems, a forced configuration) has no such epilogue.
    if (reads_a) {
        Problem p = canonical(dtype, layout, nt0 ? MG_NO_TRANS : MG_TRANS, nt0 ? MG_TRANS : MG_NO_TRANS, n, n, k, alpha, A, lda, A,
                              lda, beta, C, ldc, carve.rest(), carve.left, stream,
                              other_is_lower ? MG_SHAPE_C_UPPER : MG_SHAPE_C_LOWER);
        IndirectPlan plan;
        if (!indirect_plan(p, true, &plan)) {
            p.mask_c = true;
            const mg_status direct = run_canonical(p);
            if (direct != MG_ERR_CONFIG && direct != MG_ERR_WORKSPACE) return direct;
        }
    }
    // Otherwise the GEMM below writes all of C: the entries outside the referenced triangle are set aside first and
    // put back afterwards, bit for bit
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_copy_triangle(dtype, n, C, ldc, aside, n, other_is_lower, st) != hipSuccess) return MG_ERR_LAUNCH;
    const bool nt = trans == MG_NO_TRANS;
    // tiles wholly outside the referenced triangle are skipped (the triangle as the column-major view sees it)
    const mg_status g = run_gemm(dtype, layout, nt ? MG_NO_TRANS : MG_TRANS, nt ? MG_TRANS : MG_NO_TRANS, n, n, k, alpha, A, lda,
                                 A, lda, beta, C, ldc, carve.rest(), carve.left, stream,
                                 other_is_lower ? MG_SHAPE_C_UPPER : MG_SHAPE_C_LOWER);
    // put the other triangle back even if the product failed to launch: C is then as it was there
    if (launch_copy_triangle(dtype, n, aside, n, C, ldc, other_is_lower, st) != hipSuccess) return MG_ERR_LAUNCH;
    return g;
}

mg_status check_trmm(int layout, int side, int uplo, int trans, int diag, int64_t m, int64_t n, int64_t lda, int64_t ldb)
{
    if (layout != MG_ROW_MAJOR && layout != MG_COL_MAJOR) return MG_ERR_LAYOUT;
    if (!valid_side(side)) return MG_ERR_SIDE;
    if (!valid_uplo(uplo)) return MG_ERR_UPLO;
    if (!valid_trans(trans)) return MG_ERR_TRANS_A;
    if (!valid_diag(diag)) return MG_ERR_DIAG;
    const int64_t lim = int64_t(1) << 31;
    if (m < 0 || n < 0 || m >= lim || n >= lim) return MG_ERR_DIM;
    const int64_t ka = side == MG_LEFT ? m : n, lead = layout == MG_COL_MAJOR ? m : n;
    if (lda < (ka > 1 ? ka : 1)) return MG_ERR_LDA;
    if (ldb < (lead > 1 ? lead : 1)) return MG_ERR_LDB;
    return MG_OK;
}

mg_status run_trmm(int dtype, int layout, int side, int uplo, int trans, int diag, int64_t m, int64_t n, float alpha,
                   const void *A, int64_t lda, void *B, int64_t ldb, void *ws, size_t ws_bytes, void *stream)
{
    const mg_status s = check_trmm(layout, side, uplo, trans, diag, m, n, lda, ldb);
    if (s != MG_OK) return s;
    if (m == 0 || n == 0) return MG_OK;
    if (B == nullptr || (alpha != 0.f && A == nullptr)) return MG_ERR_NULL;
    if (alpha == 0.f) {     // B <- 0: an empty product with beta == 0
        const int64_t any = m > n ? m : n;
        return run_gemm(dtype, layout, MG_NO_TRANS, MG_NO_TRANS, m, n, 0, 0.f, nullptr, any, nullptr, any, 0.f, B, ldb,
                        nullptr, 0, stream);
    }
    const int64_t ka = side == MG_LEFT ? m : n;
    const size_t elem = dtype == MG_F32 ? 4 : 2;
    Carve carve(ws, ws_bytes);
    void *full = carve.take(static_cast<size_t>(ka) * ka * elem);
    void *copy = carve.take(static_cast<size_t>(m) * n * elem);
    if (full == nullptr || copy == nullptr) return MG_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the product cannot run in place: B is copied (tightly packed, same layout) and then overwritten; the copy and
    // the expansion of the triangular matrix go out as one launch
    const int64_t minor = layout == MG_COL_MAJOR ? m : n, major = layout == MG_COL_MAJOR ? n : m;
    if (launch_trmm_prepare(dtype, ka, A, lda, lower_in_view(layout, uplo), diag == MG_UNIT, full, minor, major, B, ldb, copy,
                            minor, st) != hipSuccess)
        return MG_ERR_LAUNCH;
    // Which canonical operand is triangular, and how: op(A) is lower when uplo and trans say so; a row-major
    // call runs as the transposed product, which swaps the operands and turns lower into upper.
    const bool op_lower = (uplo == MG_LOWER) == (trans == MG_NO_TRANS);
    const bool col = layout == MG_COL_MAJOR;
    const bool canonical_lower = col ? op_lower : !op_lower;
    const bool tri_is_a = (side == MG_LEFT) == col;
    const int shape = tri_is_a ? (canonical_lower ? MG_SHAPE_A_LOWER : MG_SHAPE_A_UPPER)
                               : (canonical_lower ? MG_SHAPE_B_LOWER : MG_SHAPE_B_UPPER);
    if (side == MG_LEFT)
        return run_gemm(dtype, layout, trans, MG_NO_TRANS, m, n, m, alpha, full, ka, copy, minor, 0.f, B, ldb, carve.rest(),
                        carve.left, stream, shape);
    return run_gemm(dtype, layout, MG_NO_TRANS, trans, m, n, n, alpha, copy, minor, full, ka, 0.f, B, ldb, carve.rest(),
                    carve.left, stream, shape);
}

}  // namespace
}  // namespace mg

using namespace mg;

// ---- the entry point that brings its own scratch memory --------------------------------------------------
// Device memory of the library itself, one copy per GPU, held until the process ends.  In host code the array's
// name is a stand-in, not a device address: the address on the current device comes from hipGetSymbolAddress,
// once per device, and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[MG_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_address[kMaxDevices] = {};
std::mutex g_scratch_mutex;

mg_status static_scratch(void **out)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return MG_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_address[device] == nullptr) {
        void *address = nullptr;
        if (hipGetSymbolAddress(&address, HIP_SYMBOL(scratch)) != hipSuccess || address == nullptr) return MG_ERR_LAUNCH;
        g_scratch_address[device] = address;
    }
    *out = g_scratch_address[device];
    return MG_OK;
}
}  // namespace

extern "C" {

mg_status mg_sgemm_static(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                          int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *stream)
{
    // what the preferred route of this problem would use (0 for invalid arguments: run_gemm names the error)
    if (mg_gemm_workspace_bytes(MG_F32, layout, ta, tb, m, n, k, lda, ldb, ldc) > MG_STATIC_SCRATCH_BYTES)
        return MG_ERR_WORKSPACE;
    void *ws = nullptr;
    const mg_status s = static_scratch(&ws);
    if (s != MG_OK) return s;
    return run_gemm(MG_F32, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, ws, MG_STATIC_SCRATCH_BYTES,
                    stream);
}

mg_status mg_sgemm(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                   int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return run_gemm(MG_F32, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, workspace,
                    workspace_bytes, stream);
}

mg_status mg_hgemm(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha, const uint16_t *A,
                   int64_t lda, const uint16_t *B, int64_t ldb, float beta, uint16_t *C, int64_t ldc,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    return run_gemm(MG_F16, layout, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, workspace,
                    workspace_bytes, stream);
}

mg_status mg_sgemv(int layout, int trans_a, int64_t m, int64_t n, float alpha, const float *A, int64_t lda,
                   const float *x, int64_t incx, float beta, float *y, int64_t incy, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return run_gemv(MG_F32, layout, trans_a, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace, workspace_bytes,
                    stream);
}

mg_status mg_hgemv(int layout, int trans_a, int64_t m, int64_t n, float alpha, const uint16_t *A, int64_t lda,
                   const uint16_t *x, int64_t incx, float beta, uint16_t *y, int64_t incy, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return run_gemv(MG_F16, layout, trans_a, m, n, alpha, A, lda, x, incx, beta, y, incy, workspace, workspace_bytes,
                    stream);
}

size_t mg_gemv_workspace_bytes(int dtype, int layout, int trans_a, int64_t m, int64_t n, int64_t lda)
{
    if (dtype != MG_F32 && dtype != MG_F16) return 0;
    if (check_gemv(layout, trans_a, m, n, lda, 1, 1) != MG_OK) return 0;
    Problem p = gemv_problem(dtype, layout, trans_a, m, n, 1.f, nullptr, lda, nullptr, 1, 1.f, nullptr, 1, nullptr,
                                   0, nullptr);
    if (p.n == 0) return 0;
    int32_t kernel = -1, split = 1;
    if (choose(p, 256, ~size_t(0), &kernel, &split) != MG_OK) return 0;
    return table()[kernel].workspace(p, split);
}

mg_status mg_sgemm_batched(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, const float *alphas,
                           const float *A, const int64_t *a_offsets, int64_t lda, const float *B,
                           const int64_t *b_offsets, int64_t ldb, const float *betas, float *C,
                           const int64_t *c_offsets, int64_t ldc, int64_t batch_count, void *stream)
{
    return generic_batched(MG_F32, layout, ta, tb, m, n, k, alphas, A, a_offsets, lda, B, b_offsets, ldb, betas, C,
                           c_offsets, ldc, batch_count, stream);
}

mg_status mg_hgemm_batched(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, const float *alphas,
                           const uint16_t *A, const int64_t *a_offsets, int64_t lda, const uint16_t *B,
                           const int64_t *b_offsets, int64_t ldb, const float *betas, uint16_t *C,
                           const int64_t *c_offsets, int64_t ldc, int64_t batch_count, void *stream)
{
    return generic_batched(MG_F16, layout, ta, tb, m, n, k, alphas, A, a_offsets, lda, B, b_offsets, ldb, betas, C,
                           c_offsets, ldc, batch_count, stream);
}

mg_status mg_sgemm_strided_batched(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha,
                                   const float *A, int64_t lda, int64_t stride_a, const float *B, int64_t ldb,
                                   int64_t stride_b, float beta, float *C, int64_t ldc, int64_t stride_c,
                                   int64_t batch_count, void *stream)
{
    return strided_batched(MG_F32, layout, ta, tb, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b, beta, C, ldc,
                           stride_c, batch_count, stream);
}

mg_status mg_hgemm_strided_batched(int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, float alpha,
                                   const uint16_t *A, int64_t lda, int64_t stride_a, const uint16_t *B, int64_t ldb,
                                   int64_t stride_b, float beta, uint16_t *C, int64_t ldc, int64_t stride_c,
                                   int64_t batch_count, void *stream)
{
    return strided_batched(MG_F16, layout, ta, tb, m, n, k, alpha, A, lda, stride_a, B, ldb, stride_b, beta, C, ldc,
                           stride_c, batch_count, stream);
}

mg_status mg_ssymm(int layout, int side, int uplo, int64_t m, int64_t n, float alpha, const float *A, int64_t lda,
                   const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *workspace, size_t workspace_bytes,
                   void *stream)
{
    return run_symm(MG_F32, layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace, workspace_bytes, stream);
}

mg_status mg_hsymm(int layout, int side, int uplo, int64_t m, int64_t n, float alpha, const uint16_t *A, int64_t lda,
                   const uint16_t *B, int64_t ldb, float beta, uint16_t *C, int64_t ldc, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return run_symm(MG_F16, layout, side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, workspace, workspace_bytes, stream);
}

mg_status mg_ssyrk(int layout, int uplo, int trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda, float beta,
                   float *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_syrk(MG_F32, layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace, workspace_bytes, stream);
}

mg_status mg_hsyrk(int layout, int uplo, int trans, int64_t n, int64_t k, float alpha, const uint16_t *A, int64_t lda,
                   float beta, uint16_t *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_syrk(MG_F16, layout, uplo, trans, n, k, alpha, A, lda, beta, C, ldc, workspace, workspace_bytes, stream);
}

mg_status mg_strmm(int layout, int side, int uplo, int trans_a, int diag, int64_t m, int64_t n, float alpha, const float *A,
                   int64_t lda, float *B, int64_t ldb, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_trmm(MG_F32, layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace, workspace_bytes, stream);
}

mg_status mg_htrmm(int layout, int side, int uplo, int trans_a, int diag, int64_t m, int64_t n, float alpha,
                   const uint16_t *A, int64_t lda, uint16_t *B, int64_t ldb, void *workspace, size_t workspace_bytes,
                   void *stream)
{
    return run_trmm(MG_F16, layout, side, uplo, trans_a, diag, m, n, alpha, A, lda, B, ldb, workspace, workspace_bytes, stream);
}

enum { MG_ROUTINE_SYMM, MG_ROUTINE_SYRK, MG_ROUTINE_TRMM };

static size_t level3_workspace_bytes(int routine, int dtype, int layout, int side, int trans, int64_t m, int64_t n, int64_t k)
{
    if (dtype != MG_F32 && dtype != MG_F16) return 0;
    if (layout != MG_ROW_MAJOR && layout != MG_COL_MAJOR) return 0;
    const int64_t lim = int64_t(1) << 31;
    if (m < 0 || n < 0 || k < 0 || m >= lim || n >= lim || k >= lim) return 0;
    const size_t elem = dtype == MG_F32 ? 4 : 2;
    const int64_t lead = layout == MG_COL_MAJOR ? m : n;
    if (routine == MG_ROUTINE_SYRK) {
        if (!valid_trans(trans) || n == 0) return 0;
        const bool nt = trans == MG_NO_TRANS;
        const int64_t la = (layout == MG_COL_MAJOR) == nt ? n : k;
        return round_up_256(static_cast<size_t>(n) * n * elem) +
               mg_gemm_workspace_bytes(dtype, layout, nt ? MG_NO_TRANS : MG_TRANS, nt ? MG_TRANS : MG_NO_TRANS, n, n, k,
                                       la > 1 ? la : 1, la > 1 ? la : 1, n);
    }
    if (!valid_side(side) || m == 0 || n == 0) return 0;
    const int64_t ka = side == MG_LEFT ? m : n;
    const size_t dense = round_up_256(static_cast<size_t>(ka) * ka * elem);
    if (routine == MG_ROUTINE_SYMM) {
        const size_t gemm = side == MG_LEFT
                                ? mg_gemm_workspace_bytes(dtype, layout, MG_NO_TRANS, MG_NO_TRANS, m, n, m, ka, lead, lead)
                                : mg_gemm_workspace_bytes(dtype, layout, MG_NO_TRANS, MG_NO_TRANS, m, n, n, lead, ka, lead);
        return dense + gemm;
    }
    if (routine == MG_ROUTINE_TRMM) {
        if (!valid_trans(trans)) return 0;
        const size_t gemm = side == MG_LEFT ? mg_gemm_workspace_bytes(dtype, layout, trans, MG_NO_TRANS, m, n, m, ka, lead, lead)
                                            : mg_gemm_workspace_bytes(dtype, layout, MG_NO_TRANS, trans, m, n, n, lead, ka, lead);
        return dense + round_up_256(static_cast<size_t>(m) * n * elem) + gemm;
    }
    return 0;
}

size_t mg_symm_workspace_bytes(int dtype, int layout, int side, int64_t m, int64_t n)
{
    return level3_workspace_bytes(MG_ROUTINE_SYMM, dtype, layout, side, MG_NO_TRANS, m, n, 0);
}

size_t mg_syrk_workspace_bytes(int dtype, int layout, int trans, int64_t n, int64_t k)
{
    return level3_workspace_bytes(MG_ROUTINE_SYRK, dtype, layout, MG_LEFT, trans, n, n, k);
}

size_t mg_trmm_workspace_bytes(int dtype, int layout, int side, int trans_a, int64_t m, int64_t n)
{
    return level3_workspace_bytes(MG_ROUTINE_TRMM, dtype, layout, side, trans_a, m, n, 0);
}

size_t mg_gemm_workspace_bytes(int dtype, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k,
                               int64_t lda, int64_t ldb, int64_t ldc)
{
    if (dtype != MG_F32 && dtype != MG_F16) return 0;
    if (check_shape(layout, ta, tb, m, n, k, lda, ldb, ldc) != MG_OK || m == 0 || n == 0) return 0;
    // scalars do not change the need except through the scale-only path, which needs none
    Problem p = canonical(dtype, layout, ta, tb, m, n, k, 1.f, nullptr, lda, nullptr, ldb, 1.f, nullptr, ldc,
                          nullptr, 0, nullptr);
    IndirectPlan plan;
    if (indirect_plan(p, false, &plan)) return plan.total();      // (the padded problem itself never splits K: it is large)
    int32_t kernel = -1, split = 1;
    if (choose(p, 256, ~size_t(0), &kernel, &split) != MG_OK) return 0;
    return table()[kernel].workspace(p, split);
}

#define MG_CONV_SHAPE_ARGS                                                                                      \
    int64_t channels, int64_t height, int64_t width, int64_t kernel_h, int64_t kernel_w, int64_t pad_h,          \
        int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dilation_h, int64_t dilation_w
#define MG_CONV_SHAPE                                                                                           \
    ConvShape { channels, height, width, kernel_h, kernel_w, pad_h, pad_w, stride_h, stride_w, dilation_h, dilation_w }

mg_status mg_sim2col(MG_CONV_SHAPE_ARGS, const float *im, float *col, void *stream)
{
    return run_im2col(MG_F32, MG_CONV_SHAPE, im, col, stream);
}

mg_status mg_him2col(MG_CONV_SHAPE_ARGS, const uint16_t *im, uint16_t *col, void *stream)
{
    return run_im2col(MG_F16, MG_CONV_SHAPE, im, col, stream);
}

mg_status mg_sconv2d(MG_CONV_SHAPE_ARGS, int64_t filters, float alpha, const float *im, const float *weights,
                     float beta, float *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_conv2d(MG_F32, MG_CONV_SHAPE, filters, alpha, im, weights, beta, out, workspace, workspace_bytes, stream);
}

mg_status mg_hconv2d(MG_CONV_SHAPE_ARGS, int64_t filters, float alpha, const uint16_t *im, const uint16_t *weights,
                     float beta, uint16_t *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_conv2d(MG_F16, MG_CONV_SHAPE, filters, alpha, im, weights, beta, out, workspace, workspace_bytes, stream);
}

size_t mg_conv2d_workspace_bytes(int dtype, MG_CONV_SHAPE_ARGS, int64_t filters)
{
    if (dtype != MG_F32 && dtype != MG_F16) return 0;
    const ConvShape s = MG_CONV_SHAPE;
    int64_t out_h, out_w, k;
    if (check_conv(s, filters, &out_h, &out_w, &k) != MG_OK || filters == 0 || out_h * out_w == 0) return 0;
    const int64_t n = out_h * out_w;
    const size_t col = conv_is_plain_gemm(s) ? 0 : round_up_256(static_cast<size_t>(k) * n * (dtype == MG_F32 ? 4 : 2));
    return col + mg_gemm_workspace_bytes(dtype, MG_ROW_MAJOR, MG_NO_TRANS, MG_NO_TRANS, filters, n, k, k, n, n);
}

int64_t mg_conv2d_out_extent(int64_t size, int64_t kernel, int64_t pad, int64_t stride, int64_t dilation)
{
    if (size < 1 || kernel < 1 || pad < 0 || stride < 1 || dilation < 1) return -1;
    return conv_out_extent(size, kernel, pad, stride, dilation);
}

int32_t mg_kernel_count(void) { return static_cast<int32_t>(table().size()); }

mg_status mg_kernel_info(int32_t kernel_id, mg_config *out)
{
    if (kernel_id < 0 || kernel_id >= mg_kernel_count() || out == nullptr) return MG_ERR_CONFIG;
    *out = table()[kernel_id].cfg;
    return MG_OK;
}

int32_t mg_lds_store_offset(int32_t k_contiguous, int32_t fragment_rows, int32_t tile_rows, int32_t row, int32_t k)
{
    if ((fragment_rows != 16 && fragment_rows != 32) || tile_rows < 64 || tile_rows > 256 || tile_rows % 64 != 0) return -1;
    if (row < 0 || row >= tile_rows || k < 0 || k >= 64) return -1;
    if (k_contiguous)
        return (fragment_rows == 16 ? mg::ldsmap::kcontig_slot<16>(row, k / 8) : mg::ldsmap::kcontig_slot<32>(row, k / 8)) + 2 * (k % 8);
    if (tile_rows < 128) return -1;
    return mg::ldsmap::transposed_slot(tile_rows, k, row / 8) + 2 * (row % 8);
}

int32_t mg_lds_read_offset(int32_t k_contiguous, int32_t fragment_rows, int32_t tile_rows, int32_t wave_row, int32_t lane,
                           int32_t fragment, int32_t k_step, int32_t half)
{
    if ((fragment_rows != 16 && fragment_rows != 32) || tile_rows < 64 || tile_rows > 256 || tile_rows % 64 != 0) return -1;
    const int steps = fragment_rows / 8;                        // K-steps per 64 values of k: 4 (32 rows) or 2
    if (wave_row < 0 || wave_row % 64 != 0 || lane < 0 || lane > 63 || fragment < 0 || k_step < 0 || k_step >= steps) return -1;
    if (wave_row + fragment_rows * (fragment + 1) > tile_rows || fragment > 7) return -1;
    if (k_contiguous) {
        if (fragment_rows == 16)
            return (mg::ldsmap::kcontig_base<16>(lane, wave_row) ^ mg::ldsmap::kcontig_xor<16>(fragment, k_step)) + fragment * 16 * 128;
        return (mg::ldsmap::kcontig_base<32>(lane, wave_row) ^ mg::ldsmap::kcontig_xor<32>(fragment, k_step)) + fragment * 32 * 128;
    }
    if (tile_rows < 128 || half < 0 || half > 1) return -1;
    const int line = 2 * tile_rows;
    const int base = fragment_rows == 16 ? (mg::ldsmap::transposed_base<16>(lane, wave_row, tile_rows) ^ mg::ldsmap::transposed_xor<16>(fragment))
                                         : (mg::ldsmap::transposed_base<32>(lane, wave_row, tile_rows) ^ mg::ldsmap::transposed_xor<32>(fragment));
    return base + k_step * (512 / fragment_rows) * line + half * 4 * line;
}

int32_t mg_lds_f32_store_offset(int32_t k_contiguous, int32_t tile_rows, int32_t row, int32_t k)
{
    if (tile_rows < 64 || tile_rows > 256 || tile_rows % 64 != 0 || row < 0 || row >= tile_rows || k < 0 || k >= 32) return -1;
    if (k_contiguous) return mg::ldsmap::kcontig_slot<32>(row, k / 4) + 4 * (k % 4);
    return mg::ldsmap::native_slot(tile_rows, k, row / 4) + 4 * (row % 4);
}

int32_t mg_lds_f32_read_offset(int32_t k_contiguous, int32_t tile_rows, int32_t wave_row, int32_t lane, int32_t fragment,
                               int32_t k_step, int32_t element)
{
    if (tile_rows < 64 || tile_rows > 256 || tile_rows % 64 != 0) return -1;
    if (wave_row < 0 || wave_row % 32 != 0 || lane < 0 || lane > 63 || fragment < 0 || k_step < 0 || k_step >= 4) return -1;
    if (wave_row + 32 * (fragment + 1) > tile_rows || element < 0 || element > 3) return -1;
    if (k_contiguous)
        return (mg::ldsmap::kcontig_base<32>(lane, wave_row) ^ mg::ldsmap::kcontig_xor<32>(fragment, k_step)) + fragment * 32 * 128 +
               4 * element;
    return mg::ldsmap::native_base(tile_rows, lane, wave_row, fragment) + (8 * k_step + element) * 4 * tile_rows;
}

const char *mg_kernel_name(int32_t kernel_id)
{
    if (kernel_id < 0 || kernel_id >= mg_kernel_count()) return "?";
    return table()[kernel_id].name;
}

mg_status mg_query_selected(int dtype, int layout, int ta, int tb, int64_t m, int64_t n, int64_t k, int64_t lda,
                            int64_t ldb, int64_t ldc, float alpha, float beta, int64_t pointer_alignment_bytes,
                            mg_config *out)
{
    if ((dtype != MG_F32 && dtype != MG_F16) || out == nullptr) return MG_ERR_CONFIG;
    mg_status s = check_shape(layout, ta, tb, m, n, k, lda, ldb, ldc);
    if (s != MG_OK) return s;
    if (m == 0 || n == 0) return MG_ERR_CONFIG;     // nothing would run
    Problem p = canonical(dtype, layout, ta, tb, m, n, k, alpha, nullptr, lda, nullptr, ldb, beta, nullptr, ldc,
                          nullptr, 0, nullptr);
    int64_t al = pointer_alignment_bytes;
    if (al <= 0 || (al & (al - 1)) != 0) return MG_ERR_CONFIG;
    if (al > 256) al = 256;
    int32_t kernel = -1, split = 1;
    s = choose(p, al, ~size_t(0), &kernel, &split);
    if (s != MG_OK) return s;
    *out = table()[kernel].cfg;
    out->split_k = split;
    out->fringe = 16 * p.fringe_m + p.fringe_n;
    return MG_OK;
}

mg_status mg_override_config(int32_t kernel_id, int32_t split_k)
{
    if (kernel_id < 0 || kernel_id >= mg_kernel_count() || split_k < 1 || split_k > 256) return MG_ERR_CONFIG;
    const KernelEntry &e = table()[kernel_id];
    if (e.launch == nullptr) return MG_ERR_CONFIG;
    g_override_kernel[e.cfg.dtype] = kernel_id;
    g_override_split[e.cfg.dtype] = split_k;
    return MG_OK;
}

mg_status mg_override_batched_config(int32_t kernel_id)
{
    if (kernel_id < 0 || kernel_id >= mg_kernel_count()) return MG_ERR_CONFIG;
    if (table()[kernel_id].launch_batched == nullptr) return MG_ERR_CONFIG;
    g_override_batched = kernel_id;
    return MG_OK;
}

mg_status mg_override_fringe(int32_t mode)
{
    if (mode != MG_FRINGE_AUTO && mode != MG_FRINGE_OFF && mode != MG_FRINGE_ON) return MG_ERR_CONFIG;
    g_fringe_mode = mode;
    return MG_OK;
}

void mg_clear_override(void)
{
    g_fringe_mode = MG_FRINGE_AUTO;
    g_override_kernel[0] = g_override_kernel[1] = -1;
    g_override_split[0] = g_override_split[1] = 1;
    g_override_batched = -1;
}

const char *mg_status_string(mg_status status)
{
    switch (status) {
        case MG_OK: return "ok";
        case MG_ERR_LAYOUT: return "invalid layout";
        case MG_ERR_TRANS_A: return "invalid transA";
        case MG_ERR_TRANS_B: return "invalid transB";
        case MG_ERR_DIM: return "negative or too large dimension";
        case MG_ERR_LDA: return "lda too small";
        case MG_ERR_LDB: return "ldb too small";
        case MG_ERR_LDC: return "ldc too small";
        case MG_ERR_NULL: return "null pointer";
        case MG_ERR_BATCH: return "invalid batch count";
        case MG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case MG_ERR_CONFIG: return "unknown or illegal kernel configuration";
        case MG_ERR_LAUNCH: return "kernel launch failed";
        case MG_ERR_NO_DEVICE: return "no usable device";
        case MG_ERR_STRIDE: return "negative batch stride";
        case MG_ERR_CONV: return "invalid convolution geometry";
        case MG_ERR_INC: return "vector increment below one";
        case MG_ERR_SIDE: return "invalid side";
        case MG_ERR_UPLO: return "invalid uplo";
        case MG_ERR_DIAG: return "invalid diag";
        default: return "unknown status";
    }
}

const char *mg_version(void) { return "0.5"; }

}  // extern "C"
