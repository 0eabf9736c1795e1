// Tucker decomposition by higher-order orthogonal iteration (Algorithm 1, section II-C) as a
// host-side driver over the contraction entry points: every tensor product of the algorithm is
// one or two single-index contractions through sb_contract, and the leading left singular
// vectors of an unfolding come from the Gram matrix of its shorter side (sb_gemm), the Jacobi
// eigensolver, and one more GEMM that maps the eigenvectors back.  Nothing synchronises with the
// host; all intermediates live in the caller's workspace.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>

#include "../../include/sbtucker.h"
#include "sb_internal.h"

hipError_t sb_eig_sym(sb_dtype dt, int n, int count, int64_t stride_bytes, void *A, void *A2, void *V, void *V2, const void *V0, void *lam, int *sel, int sweeps,
                      hipStream_t stream, void **A_final, void **V_final);
hipError_t sb_eig_gather(sb_dtype dt, int n, const void *V, const int *sel, const void *lam, int r, void *W, int64_t ldw,
                         int scaled, hipStream_t stream);
hipError_t sb_column_signs(sb_dtype dt, void *U, int64_t rows, int64_t r, int64_t ld, hipStream_t stream);
hipError_t sb_sum_slices(sb_dtype dt, const void *P, void *S, int64_t elems, int count, hipStream_t stream);

namespace {

constexpr int64_t ALIGN = 256;
int64_t esize(sb_dtype dt) { return dt == SB_F64 ? 8 : 4; }
int64_t up(int64_t bytes) { return (bytes + ALIGN - 1) / ALIGN * ALIGN; }
// cyclic Jacobi converges quadratically: random and Gram matrices of order 100-500 reach working
// precision in 6 sweeps (fp64) or 4 (fp32); the defaults leave a margin (the in-LDS solver stops
// by itself once a sweep no longer rotates anything)
int default_sweeps(sb_dtype dt, int64_t n) { return dt == SB_F64 ? (n > 128 ? 12 : 10) : (n > 128 ? 7 : 6); }

// carve-out of the workspace; sizes in bytes, every block 256-byte aligned
struct EigSpace {
    int64_t nmax;
    char *S, *S2, *V, *V2, *lam, *sel;
    static int64_t bytes(sb_dtype dt, int64_t nmax)
    {
        const int64_t mat = up(nmax * nmax * esize(dt));
        return 4 * mat + up(nmax * esize(dt)) + up(nmax * 4);
    }
    char *carve(sb_dtype dt, char *base, int64_t n)
    {
        nmax = n;
        const int64_t mat = up(n * n * esize(dt));
        S = base; S2 = S + mat; V = S2 + mat; V2 = V + mat;
        lam = V2 + mat;
        sel = lam + up(n * esize(dt));
        return sel + up(n * 4);
    }
};

// A Gram matrix of order e is a sum over `slices` slices of the tensor.  Its e x e result has few
// tiles, far fewer than the chip has compute units unless e is in the thousands, so the sum is split
// into this many partial sums (a divisor of `slices`, at most 16) that one batched call computes
// side by side and a small kernel adds up.  1: no split.
int64_t gram_parts(int64_t e, int64_t slices)
{
    const int64_t tiles = ((e + 127) / 128) * ((e + 127) / 128);
    const int64_t want = std::min<int64_t>(16, 256 / tiles);
    int64_t parts = 1;
    for (int64_t d = 2; d <= want && d <= slices; ++d)
        if (slices % d == 0) parts = d;
    return parts;
}

struct Sizes {
    int64_t m, n, p, i, j, k;
    int64_t eig_loop() const { return std::max({std::min(m, j * k), std::min(n, i * k), std::min(p, i * j)}); }
    int64_t eig_init() const { return std::max({m, n, p}); }
    // the three eigenproblems of the initialisation have the same order and are solved together
    bool init_batched() const { return m == n && n == p && m > 1; }
    int64_t rmax() const { return std::max({i, j, k}); }
    // elements of the partial Gram matrices of the initialisation (mode 1 and 2 sum over p, mode 3 over n)
    int64_t gram_elems() const
    {
        return std::max({gram_parts(m, p) * m * m, gram_parts(n, p) * n * n, gram_parts(p, n) * p * p});
    }
    int64_t y_elems() const { return std::max({m * j * k, n * i * k, i * j * p}); }
};

int64_t tucker_bytes(sb_dtype dt, const Sizes &s, int with_init)
{
    const int64_t es = esize(dt);
    const int64_t nmax = with_init ? std::max(s.eig_loop(), s.eig_init()) : s.eig_loop();
    const int64_t loop = s.eig_loop();
    return up(s.m * s.n * s.k * es) + up(s.i * s.n * s.p * es) + up(s.y_elems() * es) + up(nmax * s.rmax() * es) +
           EigSpace::bytes(dt, nmax) * (with_init && s.init_batched() ? 3 : 1) + (with_init ? up(s.gram_elems() * es) : 0) +
           4 * up(loop * loop * es);       // + previous eigenvectors of each mode, one temporary
}

struct Ctx {
    sb_dtype dt;
    hipStream_t stream;
    EigSpace eig;
    char *W;          // nmax x rmax: selected (scaled) eigenvectors
    char *Vprev[3];   // eigenvectors found for each mode in the previous iteration
    char *tmp;
    char *partial;    // partial Gram matrices of the initialisation
    bool have_prev[3];
    int warm_runs[3];    // warm starts since the last cold solve of each mode
    int status;

    bool ok() const { return status == SB_OK; }
    void check(int rc) { if (status == SB_OK && rc != SB_OK) status = rc; }
    void check_hip(hipError_t e) { if (status == SB_OK && e != hipSuccess) status = SB_ERR_LAUNCH + (int)e; }

    void gemm(sb_op ta, sb_op tb, int64_t m, int64_t n, int64_t k, const void *A, int64_t lda, const void *B, int64_t ldb,
              double beta, void *C, int64_t ldc, double alpha = 1.0)
    {
        if (!ok()) return;
        check(sb_gemm(dt, ta, tb, m, n, k, alpha, A, lda, 0, B, ldb, 0, beta, C, ldc, 0, 1, stream));
    }

    // S (e x e) = sum over q < slices of op(X_q) op(X_q)^T with X_q = X + q * step elements, each term
    // a GEMM (ta, tb) with inner extent kk and leading dimension ld.  `merge`: consecutive slices
    // continue one another along the inner index, so a run of them is one GEMM with a longer k.
    void gram(sb_op ta, sb_op tb, int64_t e, int64_t kk, bool merge, const void *X, int64_t ld, int64_t slices, int64_t step, void *S)
    {
        if (!ok()) return;
        const int64_t es = esize(dt), parts = gram_parts(e, slices), per = slices / parts;
        void *out = parts > 1 ? (void *)partial : S;
        if (merge) {
            check(sb_gemm(dt, ta, tb, e, e, kk * per, 1.0, X, ld, per * step, X, ld, per * step, 0.0, out, e, e * e, parts, stream));
        } else {
            for (int64_t t = 0; t < per && ok(); ++t) {        // partial sum g takes slices g * per + t
                const char *Xt = (const char *)X + t * step * es;
                check(sb_gemm(dt, ta, tb, e, e, kk, 1.0, Xt, ld, per * step, Xt, ld, per * step, t ? 1.0 : 0.0, out, e, e * e, parts, stream));
            }
        }
        if (parts > 1 && ok()) check_hip(sb_sum_slices(dt, partial, S, e * e, (int)parts, stream));
    }

    void contract(const char *ma, const char *mb, const char *mc, const void *A, const int64_t *dA, const void *B,
                  const int64_t *dB, void *C, const int64_t *dC)
    {
        if (!ok()) return;
        check(sb_contract(dt, ma, mb, mc, 1.0, A, dA, nullptr, B, dB, nullptr, 0.0, C, dC, nullptr, SB_AUTO, stream));
    }

    // eigenvectors of the Gram matrix already in eig.S (order e): the r leading ones go to out
    // (ld = ldo), scaled by lambda^-1/2 if `scaled`.  mode >= 0: warm start.  From one HOOI iteration
    // to the next the Gram matrix of a mode changes little, so it is first rotated by the previous
    // iteration's eigenvectors (S' = V^T S V, nearly diagonal; the Jacobi solver then stops after a
    // sweep or two) and the new eigenvectors are V V' (the solver multiplies its rotations onto V).
    void eig_leading(int mode, int64_t e, int64_t r, void *out, int64_t ldo, int scaled)
    {
        if (!ok()) return;
        const int64_t es = esize(dt);
        // The accumulated product V V' V'' ... drifts away from orthogonality by a rounding error per
        // iteration.  Every 16th solve first pulls it back with one Newton-Schulz step,
        // V <- V (3 I - V^T V) / 2, which squares the distance from orthogonality (three small GEMMs
        // instead of the five or so sweeps of a cold solve).
        const bool warm = mode >= 0 && have_prev[mode];
        if (warm && warm_runs[mode] >= 15) {
            gemm(SB_OP_T, SB_OP_N, e, e, e, Vprev[mode], e, Vprev[mode], e, 0.0, eig.V2, e);          // V^T V (solver scratch, free until the solve)
            check_hip(hipMemcpyAsync(tmp, Vprev[mode], e * e * es, hipMemcpyDeviceToDevice, stream));
            gemm(SB_OP_N, SB_OP_N, e, e, e, Vprev[mode], e, eig.V2, e, 1.5, tmp, e, -0.5);            // 1.5 V - 0.5 V (V^T V)
            std::swap(Vprev[mode], tmp);
            warm_runs[mode] = 0;
        }
        if (warm) {
            gemm(SB_OP_N, SB_OP_N, e, e, e, eig.S, e, Vprev[mode], e, 0.0, tmp, e);          // S V
            gemm(SB_OP_T, SB_OP_N, e, e, e, Vprev[mode], e, tmp, e, 0.0, eig.S, e);          // V^T (S V)
        }
        // warm: the solver's rotations accumulate onto the previous eigenvectors, so it returns V V' itself
        void *Af = nullptr, *Vf = nullptr;
        check_hip(sb_eig_sym(dt, (int)e, 1, 0, eig.S, eig.S2, eig.V, eig.V2, warm ? Vprev[mode] : nullptr, eig.lam, (int *)eig.sel,
                             default_sweeps(dt, e), stream, &Af, &Vf));
        if (!ok()) return;
        if (mode >= 0) {
            check_hip(hipMemcpyAsync(Vprev[mode], Vf, e * e * es, hipMemcpyDeviceToDevice, stream));
            if (warm) ++warm_runs[mode];
            else { have_prev[mode] = true; warm_runs[mode] = 0; }
        }
        if (!ok()) return;
        check_hip(sb_eig_gather(dt, (int)e, Vf, (const int *)eig.sel, eig.lam, (int)r, out, ldo, scaled, stream));
    }

    // U (rows x r) <- the r leading left singular vectors of the rows x R matrix Y.
    // trans == 0: Y is stored column-major with leading dimension rows;
    // trans == 1: its transpose X (R x rows, leading dimension R) is what is stored.
    void leading_left(int mode, const void *Y, int64_t rows, int64_t R, int trans, int64_t r, void *U)
    {
        const int64_t ld = trans ? R : rows;
        if (R <= rows) {                // Gram matrix of the short side: Q = Y^T Y, U = Y V_r Lambda_r^-1/2
            if (!trans) gemm(SB_OP_T, SB_OP_N, R, R, rows, Y, ld, Y, ld, 0.0, eig.S, R);
            else        gemm(SB_OP_N, SB_OP_T, R, R, rows, Y, ld, Y, ld, 0.0, eig.S, R);
            eig_leading(mode, R, r, W, R, 1);
            if (!trans) gemm(SB_OP_N, SB_OP_N, rows, r, R, Y, ld, W, R, 0.0, U, rows);
            else        gemm(SB_OP_T, SB_OP_N, rows, r, R, Y, ld, W, R, 0.0, U, rows);
        } else {                        // S = Y Y^T: its eigenvectors are the left singular vectors
            if (!trans) gemm(SB_OP_N, SB_OP_T, rows, rows, R, Y, ld, Y, ld, 0.0, eig.S, rows);
            else        gemm(SB_OP_T, SB_OP_N, rows, rows, R, Y, ld, Y, ld, 0.0, eig.S, rows);
            eig_leading(mode, rows, r, U, rows, 0);
        }
        // Singular vectors are fixed up to sign, and the sign a Jacobi solve ends with depends on its
        // path.  A fixed convention keeps each factor the same from one iteration to the next once
        // its subspace has settled, so the other modes' Gram matrices (which live in the basis of
        // these columns) stay put and their warm starts keep working.
        if (ok()) check_hip(sb_column_signs(dt, U, rows, r, rows, stream));
    }
};

}  // namespace

extern "C" int sb_tucker_workspace(sb_dtype dt, int64_t m, int64_t n, int64_t p, int64_t i, int64_t j, int64_t k,
                                   int with_init, int64_t *bytes)
{
    if (dt != SB_F64 && dt != SB_F32) return -1;
    if (m < 1) return -2;
    if (n < 1) return -3;
    if (p < 1) return -4;
    if (i < 1 || i > m || i > j * k) return -5;
    if (j < 1 || j > n || j > i * k) return -6;
    if (k < 1 || k > p || k > i * j) return -7;
    if (!bytes) return -9;
    const Sizes s{m, n, p, i, j, k};
    if (std::max(s.eig_loop(), with_init ? s.eig_init() : 0) > 4096) return -2;
    *bytes = tucker_bytes(dt, s, with_init);
    return SB_OK;
}

extern "C" int sb_tucker_hooi(sb_dtype dt, const void *T, int64_t m, int64_t n, int64_t p, int64_t i, int64_t j, int64_t k,
                              int iterations, int init, void *A, void *B, void *C, void *G, void *workspace,
                              int64_t workspace_bytes, void *stream)
{
    if (dt != SB_F64 && dt != SB_F32) return -1;
    if (m < 1) return -3;
    if (n < 1) return -4;
    if (p < 1) return -5;
    if (i < 1 || i > m || i > j * k) return -6;
    if (j < 1 || j > n || j > i * k) return -7;
    if (k < 1 || k > p || k > i * j) return -8;
    int64_t need = 0;
    if (sb_tucker_workspace(dt, m, n, p, i, j, k, init, &need) != SB_OK) return -3;      // an eigenproblem above 4096
    if (!T) return -2;
    if (iterations < 0) return -9;
    if (!A) return -11;
    if (!B) return -12;
    if (!C) return -13;
    if (!G) return -14;
    if (!workspace || (uintptr_t)workspace % ALIGN) return -15;
    if (workspace_bytes < need) return -16;

    const Sizes s{m, n, p, i, j, k};
    const int64_t es = esize(dt);
    Ctx c;
    c.dt = dt;
    c.stream = (hipStream_t)stream;
    c.status = SB_OK;
    char *w = (char *)workspace;
    char *W1 = w;  w += up(m * n * k * es);          // W1_mnk = T_mnp C_pk
    char *Z = w;   w += up(i * n * p * es);          // Z_inp  = T_mnp A_mi
    char *Y = w;   w += up(s.y_elems() * es);        // the Y of steps 4, 6, 8
    const int64_t nmax = init ? std::max(s.eig_loop(), s.eig_init()) : s.eig_loop();
    c.W = w;       w += up(nmax * s.rmax() * es);
    w = c.eig.carve(dt, w, nmax);
    const int64_t eig_bytes = EigSpace::bytes(dt, nmax);             // the same layout twice more for a batched initialisation
    if (init && s.init_batched()) w += 2 * eig_bytes;
    const int64_t loop = s.eig_loop();
    for (int q = 0; q < 3; ++q) {
        c.Vprev[q] = w;  w += up(loop * loop * es);
        c.have_prev[q] = false;
        c.warm_runs[q] = 0;
    }
    c.tmp = w;       w += up(loop * loop * es);
    c.partial = w;

    const int64_t dT[3] = {m, n, p}, dAf[2] = {m, i}, dBf[2] = {n, j}, dCf[2] = {p, k};
    const int64_t dW1[3] = {m, n, k}, dZ[3] = {i, n, p}, dY1[3] = {m, j, k}, dY2[3] = {n, i, k}, dY3[3] = {i, j, p}, dG[3] = {i, j, k};

    if (init) {
        // step 2: leading eigenvectors of T_(r) T_(r)^T.  T_(1) is the m x (np) matrix T itself,
        // T_(3)^T the (mn) x p matrix T itself; T_(2) T_(2)^T is the sum over p of T_p^T T_p.
        // A cubic tensor gives three problems of one order: they share every launch of the solver
        // (one workgroup each in LDS, or one grid row each in the multi-launch version).
        const bool batched = s.init_batched();
        char *S1 = batched ? c.eig.S + eig_bytes : c.eig.S, *S2 = batched ? c.eig.S + 2 * eig_bytes : c.eig.S;
        // Each Gram matrix is a sum over slices: frontal slices T_q (m x n) for modes 1 and 2,
        // the row blocks of T_(3)^T that belong to one value of n for mode 3.
        c.gram(SB_OP_N, SB_OP_T, m, n, true, T, m, p, m * n, c.eig.S);
        if (!batched) c.eig_leading(-1, m, i, A, m, 0);
        c.gram(SB_OP_T, SB_OP_N, n, m, false, T, m, p, m * n, S1);
        if (!batched) c.eig_leading(-1, n, j, B, n, 0);
        c.gram(SB_OP_T, SB_OP_N, p, m, true, T, m * n, n, m, S2);
        if (!batched) c.eig_leading(-1, p, k, C, p, 0);
        if (batched && c.ok()) {
            void *Af = nullptr, *Vf = nullptr;
            c.check_hip(sb_eig_sym(dt, (int)m, 3, eig_bytes, c.eig.S, c.eig.S2, c.eig.V, c.eig.V2, nullptr, c.eig.lam, (int *)c.eig.sel,
                                   default_sweeps(dt, m), c.stream, &Af, &Vf));
            void *out[3] = {A, B, C};
            const int64_t r[3] = {i, j, k};
            for (int q = 0; q < 3 && c.ok(); ++q)
                c.check_hip(sb_eig_gather(dt, (int)m, (const char *)Vf + q * eig_bytes, (const int *)(c.eig.sel + q * eig_bytes),
                                          c.eig.lam + q * eig_bytes, (int)r[q], out[q], m, 0, c.stream));
        }
    }

    for (int it = 0; it < iterations && c.ok(); ++it) {
        c.contract("mnp", "pk", "mnk", T, dT, C, dCf, W1, dW1);          // step 4: Y_mjk = T_mnp B_nj C_pk
        c.contract("mnk", "nj", "mjk", W1, dW1, B, dBf, Y, dY1);
        c.leading_left(0, Y, m, j * k, 0, i, A);                            // step 5
        c.contract("mnk", "mi", "nik", W1, dW1, A, dAf, Y, dY2);         // step 6 with mode n first: Y_(2) is a plain matrix
        c.leading_left(1, Y, n, i * k, 0, j, B);                            // step 7
        c.contract("mnp", "mi", "inp", T, dT, A, dAf, Z, dZ);            // step 8: Y_ijp = T_mnp B_nj A_mi
        c.contract("inp", "nj", "ijp", Z, dZ, B, dBf, Y, dY3);
        c.leading_left(2, Y, p, i * j, 1, k, C);                            // step 9: Y_(3) is the transpose of the (ij) x p matrix
    }
    c.contract("mnp", "mi", "inp", T, dT, A, dAf, Z, dZ);                // step 11: G_ijk = T_mnp A_mi B_nj C_pk
    c.contract("inp", "nj", "ijp", Z, dZ, B, dBf, Y, dY3);
    c.contract("ijp", "pk", "ijk", Y, dY3, C, dCf, G, dG);
    return c.status;
}

extern "C" int sb_sym_eig_workspace(sb_dtype dt, int64_t n, int64_t *bytes)
{
    if (dt != SB_F64 && dt != SB_F32) return -1;
    if (n < 1 || n > 4096) return -2;
    if (!bytes) return -3;
    *bytes = EigSpace::bytes(dt, n);
    return SB_OK;
}

extern "C" int sb_sym_eig(sb_dtype dt, int64_t n, void *S, void *V, void *lambda, int sweeps, void *workspace,
                          int64_t workspace_bytes, void *stream)
{
    int64_t need = 0;
    const int rc = sb_sym_eig_workspace(dt, n, &need);
    if (rc != SB_OK) return rc;
    if (!S) return -3;
    if (!V) return -4;
    if (!lambda) return -5;
    if (!workspace || (uintptr_t)workspace % ALIGN) return -7;
    if (workspace_bytes < need) return -8;
    EigSpace e;
    e.carve(dt, (char *)workspace, n);
    void *Af = nullptr, *Vf = nullptr;
    hipError_t err = sb_eig_sym(dt, (int)n, 1, 0, S, e.S2, e.V, e.V2, nullptr, lambda, (int *)e.sel, sweeps > 0 ? sweeps : default_sweeps(dt, n),
                                (hipStream_t)stream, &Af, &Vf);
    if (err == hipSuccess) err = sb_eig_gather(dt, (int)n, Vf, (const int *)e.sel, lambda, (int)n, V, n, 0, (hipStream_t)stream);
    return err == hipSuccess ? SB_OK : SB_ERR_LAUNCH + (int)err;
}

// ---------------------------------------------------------------------------------------------
// sb_sym_eig for callers that cannot allocate: the solver's workspace (Jacobi ping-pong copies of
// the matrix and of the eigenvectors, the eigenvalue order) lives in a file-scope device array.
// The array's name is only a host-side handle; the device address is looked up once per device
// with hipGetSymbolAddress and everything below uses that address.
namespace {

constexpr int64_t STATIC_EIG_MAX_N = SB_SYM_EIG_STATIC_MAX_N;
// EigSpace::bytes(SB_F64, 256): four 256 x 256 fp64 matrices + eigenvalues + order, each block 256-byte aligned
constexpr int64_t STATIC_EIG_BYTES = 4 * (STATIC_EIG_MAX_N * STATIC_EIG_MAX_N * 8) + STATIC_EIG_MAX_N * 8 + STATIC_EIG_MAX_N * 4;
static_assert(STATIC_EIG_MAX_N * STATIC_EIG_MAX_N * 8 % ALIGN == 0 && STATIC_EIG_MAX_N * 4 % ALIGN == 0, "blocks stay aligned");

static __device__ __align__(256) unsigned char scratch[STATIC_EIG_BYTES];

std::mutex g_scratch_lock;
void *g_scratch_ptr[SB_MAX_DEVICES] = {};

// device address of `scratch` on the current device (null + error code on failure)
hipError_t scratch_address(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= SB_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int sb_sym_eig_static(sb_dtype dt, int64_t n, void *S, void *V, void *lambda, int sweeps, void *stream)
{
    if (dt != SB_F64 && dt != SB_F32) return -1;
    if (n < 1 || n > STATIC_EIG_MAX_N) return -2;
    if (!S) return -3;
    if (!V) return -4;
    if (!lambda) return -5;
    if (EigSpace::bytes(dt, n) > STATIC_EIG_BYTES) return -2;
    void *base = nullptr;
    hipError_t err = scratch_address(&base);
    if (err != hipSuccess) return SB_ERR_LAUNCH + (int)err;
    // nothing in the workspace has to start at zero: the solver writes V (identity), the ping-pong
    // copies and the order before it reads them, so the previous call's contents are harmless
    return sb_sym_eig(dt, n, S, V, lambda, sweeps, base, STATIC_EIG_BYTES, stream);
}
