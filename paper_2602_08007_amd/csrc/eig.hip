// SVD of the k x k triangular factor R of the refresh (the "small SVD" of the randomized SVD,
// Algorithm 1's refresh step) as a chain of launches, for k <= EIG_MAXK:
//   1. T = R R^T                        fp64 MFMA GEMM, 64 x 64 tiles over the whole chip
//   2. per matrix, one workgroup:       Householder tridiagonalization of T (reflectors parked in
//      the rows of T they cleared); then eigenvalues by Sturm-count multisection (chip-wide),
//      eigenvectors of the tridiagonal matrix by inverse iteration (one per thread, pivoted LU
//      of T - lambda I), Gram-Schmidt inside groups of numerically equal eigenvalues
//   3. E = H_0 H_1 ... Z                reflectors applied to 64 eigenvectors per workgroup, the
//      vectors held in registers
//   4. E^T R                            fp64 MFMA GEMM
//   5. singular values = row norms of E^T R, ordering, fp32 outputs
// Nothing here is a serial chain longer than k steps, which is what separates it from the QL
// sweeps of the single-kernel variant (about k^2 dependent rotations per matrix).
#include <hip/hip_runtime.h>

#include "small.h"

namespace tsr {
namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
constexpr int EIG_THREADS = 1024;
constexpr int EIG_PARTS = 4;          // full-matrix pass of the tridiagonalization: pieces of a column sum
constexpr int EIG_HALF_MIN_K = 384;   // from this size on the pass moves the lower triangle only
constexpr double EIG_EPS = 2.220446049250313e-16;
// Solves per eigenvector.  With an eigenvalue good to a few ulps of the spectral radius one solve
// from a random start already carries the vector to the accuracy the gap allows (its component
// along the wanted vector is amplified by 1 / ulp relative to the others); the second covers an
// unlucky start and the third is margin (two measured 0.25 ms less per refresh of 84 matrices
// and passed every test; kept at three).
constexpr int EIG_INVIT_ROUNDS = 3;

__device__ inline double eig_wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// 1 / x to full precision for finite non-zero x of ordinary size (no scaling, no fix-up)
__device__ inline double eig_rcp(double x) {
    double r = __builtin_amdgcn_rcp(x);
    r = fma(fma(-x, r, 1.0), r, r);
    r = fma(fma(-x, r, 1.0), r, r);
    return r;
}

// Kernels that cut a matrix into chunks run one workgroup per (block b, chunk c) on a 1-D grid.
// Workgroups are handed to the eight XCDs in turn.  Chunk-major numbering spreads the chunks of
// a block over the XCDs; "pinned" numbering (block index fastest, padded to a multiple of
// eight) keeps block b on XCD b % 8, where the one-workgroup-per-block kernels also run it.
struct EigGrid { int n_blocks, chunks, pinned; };
__device__ inline bool eig_decode(const EigGrid g, int& b, int& c) {
    const int lin = blockIdx.x;
    if (g.pinned) { const int bx = (g.n_blocks + 7) / 8 * 8; b = lin % bx; c = lin / bx; }
    else { c = lin % g.chunks; b = lin / g.chunks; }
    return b < g.n_blocks && c < g.chunks;
}
inline dim3 eig_grid(const EigGrid g) {
    return dim3((unsigned)((g.pinned ? (g.n_blocks + 7) / 8 * 8 : g.n_blocks) * g.chunks));
}

// ------------------------------------------------------------------ fp64 MFMA GEMMs
// v_mfma_f64_16x16x4: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16] and receives
// D[4 v + l / 16][l % 16] in element v.  One wave owns a 32 x 32 patch (2 x 2 MFMA tiles), a
// workgroup of four waves a 64 x 64 tile; operands come straight from L2 (the matrices are a
// few hundred KB), 16 k-values per round.
// WHICH = 0: T = R R^T (R upper triangular: the sum for T[i][j] starts at max(i, j));
// WHICH = 1: E^T R into the second half of tmp (the sum for column c ends at c);
// WHICH = 2: R = R2 R1 with R2 in Gacc, both upper triangular (the sum runs from i to j).
template <int WHICH>
__global__ __launch_bounds__(256) void eig_gemm_kernel(const JacobiBlock* table, const JacobiBlock single, const EigGrid grid) {
    JacobiBlock jb = single;
    int gb, gc;
    if (!eig_decode(grid, gb, gc)) return;
    if (table) jb = table[gb];
    const JacobiBlock* blk = &jb;
    const int k = blk->k;
    const int tiles = (k + 63) >> 6;
    if (gc >= tiles * tiles) return;
    const int tm = gc / tiles, tn = gc % tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m0 = tm * 64 + (wave >> 1) * 32, n0 = tn * 64 + (wave & 1) * 32;
    if (m0 >= k || n0 >= k) return;
    const double* __restrict__ A;
    const double* __restrict__ B = (WHICH == 2) ? blk->R1 : blk->R;
    double* __restrict__ C;
    long long sam, sak, sbk, sbn;
    int k_lo = 0, k_hi = k;
    if (WHICH == 0) { A = blk->R; sam = k; sak = 1; sbk = 1; sbn = k; C = blk->tmp; k_lo = max(m0, n0) & ~3; }
    else if (WHICH == 1) { A = blk->Gacc; sam = 1; sak = k; sbk = k; sbn = 1; C = blk->tmp + (size_t)k * k; k_hi = min(k, n0 + 32); }
    else { A = blk->Gacc; sam = k; sak = 1; sbk = k; sbn = 1; C = blk->R; k_lo = m0 & ~3; k_hi = min(k, n0 + 32); }
    const int li = lane & 15, lk = lane >> 4;
    d4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};
    long long arow[2], bcol[2];
    bool aok[2], bok[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = m0 + 16 * i + li, col = n0 + 16 * i + li;
        aok[i] = row < k; bok[i] = col < k;
        arow[i] = (long long)min(row, k - 1) * sam;
        bcol[i] = (long long)min(col, k - 1) * sbn;
    }
    for (int kk = k_lo; kk < k_hi; kk += 16) {
        double a[4][2], b[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int kc = kk + 4 * u + lk;
            const bool kok = kc < k_hi;
            const long long kcc = min(kc, k - 1);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const double av = A[arow[i] + kcc * sak];
                const double bv = B[kcc * sbk + bcol[i]];
                a[u][i] = (kok && aok[i]) ? av : 0.0;
                b[u][i] = (kok && bok[i]) ? bv : 0.0;
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u][i], b[u][j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + 16 * i + 4 * v + lk, col = n0 + 16 * j + li;
                if (row < k && col < k) C[(size_t)row * k + col] = acc[i][j][v];
            }
}

// ------------------------------------------------------------------ tridiagonal eigenproblem
// Start vector of the inverse iteration: a fixed pseudo-random value in (-0.5, 0.5) per entry
// (integer finalizer of the published MurmurHash3).
__device__ inline double eig_start_value(unsigned i, unsigned j) {
    unsigned h = i * 2654435761u ^ (j * 40503u + 0x9E3779B9u);
    h ^= h >> 16; h *= 0x85EBCA6Bu; h ^= h >> 13; h *= 0xC2B2AE35u; h ^= h >> 16;
    return (double)h * (1.0 / 4294967296.0) - 0.5 + 1.0 / 8589934592.0;
}

__global__ __launch_bounds__(EIG_THREADS) void eig_tridiag_kernel(const JacobiBlock* table, const JacobiBlock single) {
    JacobiBlock jb = single;
    if (table) jb = table[blockIdx.x];
    const JacobiBlock* blk = &jb;
    const int k = blk->k;
    double* T = blk->tmp;                       // symmetric, full storage; afterwards the reflectors
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double s_d[EIG_MAXK];            // diagonal
    __shared__ double s_e[EIG_MAXK];            // sub-diagonal, s_e[i] couples i and i + 1
    __shared__ double s_v[EIG_MAXK];            // Householder vector v and companion w of two
    __shared__ double s_w[EIG_MAXK];            //   consecutive reflectors (pending / being formed)
    __shared__ double s_vn[EIG_MAXK];
    __shared__ double s_wn[EIG_MAXK];
    __shared__ double s_part[(EIG_THREADS / 128) * EIG_MAXK];   // column sums of the waves, two waves per slot
    __shared__ double s_prow[EIG_MAXK];                         // row sums
    __shared__ double s_red[EIG_THREADS / 64];

    auto block_sum = [&](double v) -> double {
        v = eig_wave_sum(v);
        __syncthreads();
        if (lane == 0) s_red[wave] = v;
        __syncthreads();
        double t = 0.0;
        for (int i = 0; i < nw; ++i) t += s_red[i];
        return t;
    };

    // ---- Householder tridiagonalization.  Reflector t, H_t = I - beta v v^T on indices
    // t+1..k-1, clears column t below the sub-diagonal; v goes to row t of T (columns t+1..),
    // beta to T[t][t].  The rank-two update of reflector t-1,  T -= v w^T + w v^T, is still
    // pending when reflector t is formed: column t is corrected on the fly, and one pass over
    // the trailing matrix then applies the pending update and multiplies the updated matrix
    // with the new v.  The pass runs at the rate one CU moves data to and from L2.  Small
    // matrices (k < EIG_HALF_MIN_K) keep the full symmetric matrix up to date: a thread owns a
    // piece of a column, whose sum has one target.  Larger ones keep and move the lower
    // triangle only (half the matrix, half the time; for small ones the short rows make that
    // form the slower one): the rows are dealt to the waves in turn, a wave sweeps its row up to the
    // diagonal in strips of 64 columns, and an entry (c, i) below the diagonal adds to two sums
    // of p = T v, p_i (kept per lane and strip over all rows of the wave, summed over the waves
    // through LDS at the end) and p_c (summed over the lanes once per row); the upper triangle
    // is then dead storage from the first pass on.  Either way row t receives reflector t.
    // (v, w) are indexed from t for the pending pair and from t+1 for the new one.
    constexpr int STRIPS = (EIG_MAXK + 63) / 64;
    const bool half = k >= EIG_HALF_MIN_K;
    const int parts = EIG_PARTS;
    const int tpp = nt / parts;
    const int part = tid / tpp, li = tid % tpp;
    for (int i = tid; i < k; i += nt) { s_v[i] = 0.0; s_w[i] = 0.0; }
    __syncthreads();
    double* pv_ = s_v; double* pw_ = s_w;      // pending pair
    double* nv_ = s_vn; double* nw_ = s_wn;    // pair being formed
    for (int t = 0; t + 2 < k; ++t) {
        const int n1 = k - t - 1;
        const double v0 = pv_[0], w0 = pw_[0];
        // column t below the diagonal; with the full matrix kept, read along row t (coalesced)
        double psum = 0.0;
        for (int i = tid; i < n1; i += nt) {
            const double tc = half ? T[(size_t)(t + 1 + i) * k + t] : T[(size_t)t * k + t + 1 + i];
            const double x = tc - v0 * pw_[1 + i] - w0 * pv_[1 + i];
            nv_[i] = x;
            psum += x * x;
        }
        const double dnew = T[(size_t)t * k + t] - 2.0 * v0 * w0;
        const double xnorm2 = block_sum(psum);
        const double x0 = nv_[0];
        const double xn = sqrt(xnorm2);
        double alpha = (x0 >= 0.0) ? -xn : xn;
        const double vnorm2 = xnorm2 - 2.0 * alpha * x0 + alpha * alpha;     // |x - alpha e1|^2
        const bool skip = (xnorm2 - x0 * x0 <= 0.0) || vnorm2 <= 0.0;        // already tridiagonal here
        if (skip) alpha = x0;
        const double beta = skip ? 0.0 : 2.0 / vnorm2;
        __syncthreads();
        if (tid == 0) { s_d[t] = dnew; s_e[t] = alpha; T[(size_t)t * k + t] = beta; nv_[0] = x0 - alpha; }
        if (skip) { for (int i = tid; i < n1; i += nt) nv_[i] = 0.0; }       // no reflector: only the pending update runs
        __syncthreads();
        if (!skip) { for (int i = tid; i < n1; i += nt) T[(size_t)t * k + t + 1 + i] = nv_[i]; }
        double pv = 0.0;
        if (half) {
            // entry (c, i), i <= c, of the trailing matrix: pending update, then its terms of p = T v
            double colacc[STRIPS];
#pragma unroll
            for (int q = 0; q < STRIPS; ++q) colacc[q] = 0.0;
            // (the next row of a wave is fetched while the current one is worked on)
            auto fetch = [&](int c, double* x) {
                const double* row = T + (size_t)(t + 1 + c) * k + (t + 1);
#pragma unroll
                for (int q = 0; q < STRIPS; ++q) {
                    const int i = 64 * q + lane;
                    x[q] = (c < n1 && i <= c) ? row[i] : 0.0;
                }
            };
            double xa[STRIPS], xb[STRIPS];
            fetch(wave, xa);
            auto work = [&](int c, const double* x) {
                const double vc = pv_[1 + c], wc = pw_[1 + c], nc = nv_[c];
                double* row = T + (size_t)(t + 1 + c) * k + (t + 1);
                double rowacc = 0.0;
#pragma unroll
                for (int q = 0; q < STRIPS; ++q) {
                    const int i = 64 * q + lane;
                    if (i <= c) {
                        const double xi = x[q] - (vc * pw_[1 + i] + wc * pv_[1 + i]);
                        row[i] = xi;
                        colacc[q] += xi * nc;
                        if (i < c) rowacc += xi * nv_[i];
                    }
                }
                rowacc = eig_wave_sum(rowacc);
                if (lane == 0) s_prow[c] = rowacc;
            };
            for (int c = wave; c < n1; c += 2 * nw) {
                fetch(c + nw, xb);
                work(c, xa);
                if (c + nw < n1) {
                    fetch(c + 2 * nw, xa);
                    work(c + nw, xb);
                }
            }
            // column sums of the waves: the first half of the waves store theirs, the second half add to them
            if (wave < nw / 2) {
#pragma unroll
                for (int q = 0; q < STRIPS; ++q)
                    if (64 * q + lane < n1) s_part[wave * EIG_MAXK + 64 * q + lane] = colacc[q];
            }
            __syncthreads();
            if (wave >= nw / 2) {
#pragma unroll
                for (int q = 0; q < STRIPS; ++q)
                    if (64 * q + lane < n1) s_part[(wave - nw / 2) * EIG_MAXK + 64 * q + lane] += colacc[q];
            }
            __syncthreads();
            for (int i = tid; i < n1; i += nt) {
                double a = s_prow[i];
                for (int q = 0; q < nw / 2; ++q) a += s_part[q * EIG_MAXK + i];
                a *= beta;
                nw_[i] = a;
                pv += a * nv_[i];
            }
        } else {
            const int seg = (n1 + parts - 1) / parts;
            const int c_lo = min(n1, part * seg), c_hi = min(n1, c_lo + seg);
            // entry (c, i) of the trailing matrix, c in this thread's piece: pending update, then its
            // term of p = T v (rows read as columns, coalesced over the output index i)
            for (int i = li; i < n1; i += tpp) {
                const double vi = pv_[1 + i], wi = pw_[1 + i];
                double acc[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
                double* col = T + (size_t)(t + 1) * k + (t + 1 + i);
                int c = c_lo;
                for (; c + 8 <= c_hi; c += 8) {
                    double x[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) x[u] = col[(size_t)(c + u) * k];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        x[u] -= pv_[1 + c + u] * wi + pw_[1 + c + u] * vi;
                        col[(size_t)(c + u) * k] = x[u];
                        acc[u] += x[u] * nv_[c + u];
                    }
                }
                for (; c < c_hi; ++c) {
                    const double x = col[(size_t)c * k] - (pv_[1 + c] * wi + pw_[1 + c] * vi);
                    col[(size_t)c * k] = x;
                    acc[0] += x * nv_[c];
                }
                s_part[part * EIG_MAXK + i] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
            }
            __syncthreads();
            for (int i = tid; i < n1; i += nt) {
                double a = 0.0;
                for (int q = 0; q < parts; ++q) a += s_part[q * EIG_MAXK + i];
                a *= beta;
                nw_[i] = a;
                pv += a * nv_[i];
            }
        }
        const double kk2 = 0.5 * beta * block_sum(pv);
        for (int i = tid; i < n1; i += nt) nw_[i] -= kk2 * nv_[i];           // w = p - (beta/2)(p.v) v
        __syncthreads();
        double* sw;
        sw = pv_; pv_ = nv_; nv_ = sw;
        sw = pw_; pw_ = nw_; nw_ = sw;
    }
    // the last pending update touches the trailing 2 x 2 block only
    if (tid == 0) {
        if (k >= 2) {
            s_d[k - 2] = T[(size_t)(k - 2) * k + k - 2] - 2.0 * pv_[0] * pw_[0];
            s_e[k - 2] = T[(size_t)(k - 1) * k + k - 2] - pv_[1] * pw_[0] - pw_[1] * pv_[0];
            s_d[k - 1] = T[(size_t)(k - 1) * k + k - 1] - 2.0 * pv_[1] * pw_[1];
        } else {
            s_d[0] = T[0];
        }
        s_e[k - 1] = 0.0;
    }
    __syncthreads();
    // the tridiagonal matrix travels to the next launch behind the LU scratch
    double* DE = blk->scratch + (size_t)3 * k * k;
    for (int i = tid; i < k; i += nt) { DE[i] = s_d[i]; DE[k + i] = s_e[i]; }
}

// Eigenvalues and eigenvectors of the tridiagonal matrix (d, e) left by eig_tridiag_kernel, in
// three launches: eigenvalues (chip-wide), inverse iteration (one wave per workgroup),
// orthogonalisation inside groups of numerically equal eigenvalues (one workgroup per matrix).
// Behind the LU scratch (3 k^2 doubles) sit d (k), e (k), the eigenvalues (k, ascending) and the
// radius of the spectrum's bracket (1; zero marks a zero or non-finite matrix).

// Sturm-count multisection: 32 eigenvalues per workgroup, 8 threads each; 7 probes cut an
// eigenvalue's bracket into 8 pieces per pass, and the number of eigenvalues below a probe
// tells on which side of it the wanted one lies.
constexpr int EIG_VAL_PER_WG = 32;
__global__ __launch_bounds__(256) void eig_values_kernel(const JacobiBlock* table, const JacobiBlock single, const EigGrid grid) {
    JacobiBlock jb = single;
    int gb, gc;
    if (!eig_decode(grid, gb, gc)) return;
    if (table) jb = table[gb];
    const JacobiBlock* blk = &jb;
    const int k = blk->k;
    const int e0 = gc * EIG_VAL_PER_WG;
    if (e0 >= k) return;
    const double* DE = blk->scratch + (size_t)3 * k * k;
    double* LAM = blk->scratch + (size_t)3 * k * k + 2 * k;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double s_d[EIG_MAXK];            // diagonal
    __shared__ double s_w[EIG_MAXK];            // squared sub-diagonal
    __shared__ double s_lo[EIG_VAL_PER_WG];     // eigenvalue brackets
    __shared__ double s_hi[EIG_VAL_PER_WG];
    __shared__ int s_cnt[256];                  // Sturm counts of the probes
    __shared__ double s_red[4];
    auto block_max = [&](double v) -> double {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
        __syncthreads();
        if (lane == 0) s_red[wave] = v;
        __syncthreads();
        double t = s_red[0];
        for (int i = 1; i < nw; ++i) t = fmax(t, s_red[i]);
        return t;
    };
    double gl = 0.0, gu = 0.0;
    {
        double lo = 1e300, hi = -1e300;
        for (int i = tid; i < k; i += nt) {
            const double di = DE[i], ei = DE[k + i];
            const double rad = ((i > 0) ? fabs(DE[k + i - 1]) : 0.0) + ((i < k - 1) ? fabs(ei) : 0.0);
            lo = fmin(lo, di - rad);
            hi = fmax(hi, di + rad);
            s_d[i] = di;
            s_w[i] = ei * ei;
        }
        gu = block_max(hi);
        gl = -block_max(-lo);
    }
    double tnorm = fmax(fabs(gl), fabs(gu));
    const bool degenerate = !(tnorm > 0.0) || !(tnorm < 1e300);   // zero (or non-finite) matrix
    if (degenerate) tnorm = 0.0;
    if (gc == 0 && tid == 0) LAM[k] = tnorm;
    if (degenerate) {
        if (tid < EIG_VAL_PER_WG && e0 + tid < k) LAM[e0 + tid] = 0.0;
        return;
    }
    const double pivmin = fmax(1e-290, 1e-32 * tnorm);
    {
        const double margin = 2.0 * EIG_EPS * tnorm * (double)k + 2.0 * pivmin;
        gl -= margin; gu += margin;
    }
    constexpr int S = 7;
    const int el = tid >> 3, es = tid & 7;
    const int ej = e0 + el;
    const bool eact = ej < k && es < S;
    int passes = 0;
    for (double shrink = 1.0; shrink < 1.5e17; shrink *= (double)(S + 1)) ++passes;       // 2^-57 of the bracket
    if (tid < EIG_VAL_PER_WG) { s_lo[tid] = gl; s_hi[tid] = gu; }
    __syncthreads();
    const double inv_pieces = 1.0 / (double)(S + 1);
    for (int pass = 0; pass < passes; ++pass) {
        if (eact) {
            const double lo = s_lo[el], hi = s_hi[el];
            const double x = lo + (double)(es + 1) * ((hi - lo) * inv_pieces);
            double q = s_d[0] - x;
            if (fabs(q) < pivmin) q = -pivmin;
            int cnt = (q < 0.0) ? 1 : 0;
            for (int i = 1; i < k; ++i) {
                q = (s_d[i] - x) - s_w[i - 1] * eig_rcp(q);
                if (fabs(q) < pivmin) q = -pivmin;
                cnt += (q < 0.0) ? 1 : 0;
            }
            s_cnt[tid] = cnt;
        }
        __syncthreads();
        if (eact && es == 0) {
            const double lo = s_lo[el], hi = s_hi[el];
            const double step = (hi - lo) * inv_pieces;
            int m = 0;                                       // leading probes at or below eigenvalue ej
            while (m < S && s_cnt[tid + m] <= ej) ++m;
            if (m > 0) s_lo[el] = lo + (double)m * step;
            if (m < S) s_hi[el] = lo + (double)(m + 1) * step;
        }
        __syncthreads();
    }
    if (tid < EIG_VAL_PER_WG && e0 + tid < k) LAM[e0 + tid] = 0.5 * (s_lo[tid] + s_hi[tid]);
}

// Eigenvectors by inverse iteration, vector j on its own thread, one wave per workgroup (the
// recurrences are serial in the row index and wait on L2 for their operands: a wave alone on
// its SIMD; up to sixteen rows are fetched at a time).  T - lambda I = P L U with
// partial pivoting; U (three diagonals, pivots as reciprocals) is kept, L is applied to the
// right-hand side while it is formed and formed again in every round.
__global__ __launch_bounds__(64) void eig_invit_kernel(const JacobiBlock* table, const JacobiBlock single, const EigGrid grid) {
    JacobiBlock jb = single;
    int gb, gc;
    if (!eig_decode(grid, gb, gc)) return;
    if (table) jb = table[gb];
    const JacobiBlock* blk = &jb;
    const int k = blk->k;
    if (gc * 64 >= k) return;
    double* Z = blk->tmp + (size_t)k * k;       // eigenvectors of the tridiagonal matrix, Z[i][j] = j-th vector
    double* U0 = blk->scratch;                  // per thread j: reciprocal pivots, first and second
    double* U1 = U0 + (size_t)k * k;            //   super-diagonal of the LU factor, entry [i][j]
    double* U2 = U1 + (size_t)k * k;
    const double* DE = blk->scratch + (size_t)3 * k * k;
    const double* LAM = DE + 2 * k;
    const int tid = threadIdx.x;
    const int j = gc * 64 + tid;
    __shared__ double s_d[EIG_MAXK];            // diagonal
    __shared__ double s_e[EIG_MAXK];            // sub-diagonal, s_e[i] couples i and i + 1
    for (int i = tid; i < k; i += 64) { s_d[i] = DE[i]; s_e[i] = DE[k + i]; }
    __syncthreads();
    const double tnorm = LAM[k];
    if (tnorm == 0.0) {
        // zero (or non-finite) matrix: every orthonormal basis is one of eigenvectors
        if (j < k) for (int i = 0; i < k; ++i) Z[(size_t)i * k + j] = (i == j) ? 1.0 : 0.0;
        return;
    }
    const double tiny = EIG_EPS * tnorm;                 // floor of an LU pivot
    int vz;                                              // a zero the compiler keeps in a vector register
    asm volatile("v_mov_b32 %0, 0" : "=v"(vz));
    if (j < k) {
        const double lam = LAM[j];
        double* zc = Z + j;
        double* u0 = U0 + j; double* u1 = U1 + j; double* u2 = U2 + j;
        double scale = 1.0;
        for (int round = 0; round < EIG_INVIT_ROUNDS; ++round) {
            // forward: eliminate, apply to y (first time round: the start vector, later scale * previous x)
            auto yval = [&](int i) -> double {
                return (round == 0) ? eig_start_value((unsigned)i, (unsigned)j) : scale * zc[(size_t)i * k];
            };
            double a = s_d[0] - lam, b = (k > 1) ? s_e[0] : 0.0;
            double ycur = yval(0);
            auto step = [&](int i, double ynext) {
                const double c = s_e[i];
                const double dn = s_d[i + 1] - lam;
                const double en = (i + 2 < k) ? s_e[i + 1] : 0.0;
                const size_t o = (size_t)i * k;
                if (fabs(a) >= fabs(c)) {
                    double piv = a;
                    if (fabs(piv) < tiny) piv = (piv < 0.0) ? -tiny : tiny;
                    const double inv = eig_rcp(piv);
                    const double mult = c * inv;
                    if (round == 0) { u0[o] = inv; u1[o] = b; u2[o] = 0.0; }
                    zc[o] = ycur;
                    a = dn - mult * b; b = en;
                    ycur = ynext - mult * ycur;
                } else {
                    double piv = c;
                    if (fabs(piv) < tiny) piv = (piv < 0.0) ? -tiny : tiny;
                    const double inv = eig_rcp(piv);
                    const double mult = a * inv;
                    if (round == 0) { u0[o] = inv; u1[o] = dn; u2[o] = en; }
                    zc[o] = ynext;
                    a = b - mult * dn; b = -mult * en;
                    ycur = ycur - mult * ynext;
                }
            };
            {
                int i = 0;
                for (; i + 16 < k; i += 16) {                // rows i+1 .. i+16 fetched together
                    double yn[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u) yn[u] = yval(i + 1 + u);
#pragma unroll
                    for (int u = 0; u < 16; ++u) step(i + u, yn[u]);
                }
                for (; i + 1 < k; ++i) step(i, yval(i + 1));
            }
            {
                double piv = a;
                if (fabs(piv) < tiny) piv = (piv < 0.0) ? -tiny : tiny;
                if (round == 0) { u0[(size_t)(k - 1) * k] = eig_rcp(piv); u1[(size_t)(k - 1) * k] = 0.0; u2[(size_t)(k - 1) * k] = 0.0; }
                zc[(size_t)(k - 1) * k] = ycur;
            }
            // backward: U x = y, sixteen rows fetched together (row offsets kept in vector registers:
            // as wave-uniform values they would need more scalar registers than there are)
            double x1 = 0.0, x2 = 0.0, amax = 0.0;      // x[i+1], x[i+2]
            bool bad = false;
            int i = k - 1;
            for (; i >= 15; i -= 16) {
                double y[16], p0[16], p1[16], p2[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const size_t o = (size_t)(i - u + vz) * k;
                    y[u] = zc[o]; p0[u] = u0[o]; p1[u] = u1[o]; p2[u] = u2[o];
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const double x = (y[u] - p1[u] * x1 - p2[u] * x2) * p0[u];
                    zc[(size_t)(i - u) * k] = x;
                    amax = fmax(amax, fabs(x));
                    bad = bad || !(fabs(x) <= 1e300);
                    x2 = x1; x1 = x;
                }
            }
            for (; i >= 0; --i) {
                const size_t o = (size_t)i * k;
                const double x = (zc[o] - u1[o] * x1 - u2[o] * x2) * u0[o];
                zc[o] = x;
                amax = fmax(amax, fabs(x));
                bad = bad || !(fabs(x) <= 1e300);
                x2 = x1; x1 = x;
            }
            if (bad || !(amax > 0.0)) {
                // overflow or a vanished vector (the floored pivots are meant to rule both out):
                // go on from the unit vector rather than carry a non-finite value
                for (int q = 0; q < k; ++q) zc[(size_t)q * k] = (q == j) ? 1.0 : 0.0;
                amax = 1.0;
            }
            scale = 1.0 / amax;
        }
        double ss = 0.0;
        for (int i = 0; i < k; ++i) { const double x = scale * zc[(size_t)i * k]; ss += x * x; }
        const double nrm = scale / sqrt(ss);
        for (int i = 0; i < k; ++i) zc[(size_t)i * k] *= nrm;
    }
}

// Eigenvalues closer than ortol form a group; inside a group the vectors of the inverse
// iteration span the right subspace but need not be orthogonal: Gram-Schmidt (two passes) in
// order.  One workgroup per matrix; returns at once when there is no group.
__global__ __launch_bounds__(EIG_THREADS) void eig_groups_kernel(const JacobiBlock* table, const JacobiBlock single) {
    JacobiBlock jb = single;
    if (table) jb = table[blockIdx.x];
    const JacobiBlock* blk = &jb;
    const int k = blk->k;
    double* Z = blk->tmp + (size_t)k * k;
    const double* LAM = blk->scratch + (size_t)3 * k * k + 2 * k;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double s_v[EIG_MAXK];            // eigenvalues, ascending
    __shared__ double s_part[EIG_MAXK];         // Gram-Schmidt coefficients
    __shared__ double s_red[EIG_THREADS / 64];
    __shared__ int s_first[EIG_MAXK];           // first member of the group an eigenvalue belongs to
    __shared__ int s_any;
    auto block_sum = [&](double v) -> double {
        v = eig_wave_sum(v);
        __syncthreads();
        if (lane == 0) s_red[wave] = v;
        __syncthreads();
        double t = 0.0;
        for (int i = 0; i < nw; ++i) t += s_red[i];
        return t;
    };
    const double tnorm = LAM[k];
    if (tnorm == 0.0) return;
    if (tid == 0) s_any = 0;
    for (int i = tid; i < k; i += nt) s_v[i] = LAM[i];
    __syncthreads();
    {
        const double ortol0 = 1e-9 * tnorm;
        for (int i = 1 + tid; i < k; i += nt) if (s_v[i] - s_v[i - 1] <= ortol0) s_any = 1;
    }
    __syncthreads();
    if (s_any == 0) return;
    // ---- eigenvalues closer than ortol form a group; inside a group the vectors found above
    // span the right subspace but need not be orthogonal: Gram-Schmidt (two passes) in order.
    {
        const double ortol = 1e-9 * tnorm;
        if (tid == 0) {
            s_first[0] = 0;
            for (int j = 1; j < k; ++j) s_first[j] = (s_v[j] - s_v[j - 1] <= ortol) ? s_first[j - 1] : j;
        }
        __syncthreads();
        double* coef = s_part;
        for (int j = 1; j < k; ++j) {
            const int cs = s_first[j];
            if (cs == j) continue;                       // uniform
            for (int pass = 0; pass < 2; ++pass) {
                for (int i = cs + wave; i < j; i += nw) {
                    double a = 0.0;
                    for (int t = lane; t < k; t += 64) a += Z[(size_t)t * k + i] * Z[(size_t)t * k + j];
                    a = eig_wave_sum(a);
                    if (lane == 0) coef[i - cs] = a;
                }
                __syncthreads();
                for (int t = tid; t < k; t += nt) {
                    double a = 0.0;
                    for (int i = cs; i < j; ++i) a += coef[i - cs] * Z[(size_t)t * k + i];
                    Z[(size_t)t * k + j] -= a;
                }
                __syncthreads();
            }
            double ss = 0.0;
            for (int t = tid; t < k; t += nt) { const double x = Z[(size_t)t * k + j]; ss += x * x; }
            ss = block_sum(ss);
            const double inv = (ss > 0.0) ? 1.0 / sqrt(ss) : 0.0;
            for (int t = tid; t < k; t += nt) Z[(size_t)t * k + j] *= inv;
            __syncthreads();
        }
    }
}

// ------------------------------------------------------------------ back-transformation
// E = H_0 H_1 ... H_{k-3} Z for 64 columns of Z per workgroup: lane = column, each of the WAVES
// waves owns EPT consecutive rows (in registers); the reflector entries are uniform over a
// wave.  One barrier per reflector (the dot product spans the waves).
template <int EPT, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void eig_backtransform_kernel(const JacobiBlock* table, const JacobiBlock single, const EigGrid grid) {
    JacobiBlock jb = single;
    int gb, gc;
    if (!eig_decode(grid, gb, gc)) return;
    if (table) jb = table[gb];
    const JacobiBlock* blk = &jb;
    const int k = blk->k;
    const int c0 = gc * 64;
    if (c0 >= k) return;
    typedef const double __attribute__((address_space(1))) gdouble;
    typedef double d8 __attribute__((ext_vector_type(8)));
    typedef d8 __attribute__((aligned(8))) d8u;
    typedef const d8u __attribute__((address_space(1))) cd8u;
    static_assert(EPT % 8 == 0, "rows per wave come in chunks of eight");
    // the reflector entries have wave-uniform addresses: they travel through the scalar data path
    const gdouble* __restrict__ T = (const gdouble*)blk->tmp;
    const double* __restrict__ Z = blk->tmp + (size_t)k * k;
    double* __restrict__ E = blk->Gacc;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = c0 + lane;
    const bool colok = col < k;
    const int i0 = wave * EPT;
    __shared__ double s_dot[2][WAVES][64];
    double x[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const int i = i0 + e;
        x[e] = (colok && i < k) ? Z[(size_t)min(i, k - 1) * k + min(col, k - 1)] : 0.0;
    }
    int par = 0;
    for (int j = k - 3; j >= 0; --j) {
        const double beta = T[(size_t)j * k + j];
        if (beta == 0.0) continue;                          // uniform: no reflector at this step
        const gdouble* __restrict__ vrow = T + (size_t)j * k;
        const bool active = i0 + EPT > j + 1 && i0 < k;     // uniform over the wave
        // eight reflector entries per fetch; chunks that end at or before j hold no entry of v.
        // (A chunk may reach past column k-1: what it reads there is still inside tmp, which
        // carries 64 doubles of padding for the smallest k, and is masked out.)
        double part = 0.0;
        if (active) {
#pragma unroll
            for (int c = 0; c < EPT / 8; ++c) {
                const int ib = i0 + 8 * c;
                if (ib > j && ib + 7 < k) {                 // whole chunk inside the reflector
                    const d8u v8 = *(const cd8u*)(vrow + ib);
#pragma unroll
                    for (int u = 0; u < 8; ++u) part += v8[u] * x[8 * c + u];
                } else if (ib + 7 > j && ib < k) {
                    const d8u v8 = *(const cd8u*)(vrow + ib);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const double v = (ib + u > j && ib + u < k) ? v8[u] : 0.0;
                        part += v * x[8 * c + u];
                    }
                }
            }
        }
        s_dot[par][wave][lane] = part;
        __syncthreads();
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) tot += s_dot[par][w][lane];
        const double s = beta * tot;
        if (active) {
#pragma unroll
            for (int c = 0; c < EPT / 8; ++c) {
                const int ib = i0 + 8 * c;
                if (ib > j && ib + 7 < k) {
                    const d8u v8 = *(const cd8u*)(vrow + ib);
#pragma unroll
                    for (int u = 0; u < 8; ++u) x[8 * c + u] -= s * v8[u];
                } else if (ib + 7 > j && ib < k) {
                    const d8u v8 = *(const cd8u*)(vrow + ib);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const double v = (ib + u > j && ib + u < k) ? v8[u] : 0.0;
                        x[8 * c + u] -= s * v;
                    }
                }
            }
        }
        par ^= 1;
    }
    if (colok) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int i = i0 + e;
            if (i < k) E[(size_t)i * k + col] = x[e];
        }
    }
}

// ------------------------------------------------------------------ ordering and outputs
// Rows of E^T R (second half of tmp) are mutually orthogonal with norms sigma_i.
__global__ __launch_bounds__(EIG_THREADS) void eig_finish_kernel(const JacobiBlock* table, const JacobiBlock single) {
    JacobiBlock jb = single;
    if (table) jb = table[blockIdx.x];
    const JacobiBlock* blk = &jb;
    const int k = blk->k, r = blk->r;
    const double* __restrict__ ER = blk->tmp + (size_t)k * k;
    const double* __restrict__ E = blk->Gacc;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nt >> 6;
    __shared__ double s_sig[EIG_MAXK];
    __shared__ int s_rank[EIG_MAXK];
    for (int j = wave; j < k; j += nw) {
        double a = 0.0;
        for (int c = lane; c < k; c += 64) { const double v = ER[(size_t)j * k + c]; a += v * v; }
        a = eig_wave_sum(a);
        if (lane == 0) s_sig[j] = sqrt(a);
    }
    __syncthreads();
    for (int j = tid; j < k; j += nt) {
        const double sj = s_sig[j];
        int rank = 0;
        for (int i = 0; i < k; ++i) {
            const double si = s_sig[i];
            rank += (si > sj || (si == sj && i < j)) ? 1 : 0;
        }
        s_rank[j] = rank;
        if (blk->sigma) blk->sigma[rank] = (float)sj;
    }
    __syncthreads();
    for (int j = wave; j < k; j += nw) {
        const int rank = s_rank[j];
        if (rank >= r) continue;
        const double sj = s_sig[j];
        const double inv = (sj > 0.0) ? 1.0 / sj : 0.0;
        for (int c = lane; c < k; c += 64) {
            blk->XrT[(size_t)rank * k + c] = (float)(ER[(size_t)j * k + c] * inv);
            blk->GrT[(size_t)rank * k + c] = (float)E[(size_t)c * k + j];
        }
    }
}

}  // namespace

hipError_t launch_rtot_product(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                               hipStream_t stream) {
    if (blocks <= 0 || max_k < 1) return hipSuccess;
    JacobiBlock sb{};
    if (single) sb = *single;
    const int tiles = (max_k + 63) / 64;
    const EigGrid gt{blocks, tiles * tiles, 0};
    hipLaunchKernelGGL(eig_gemm_kernel<2>, eig_grid(gt), dim3(256), 0, stream, table_dev, sb, gt);
    return hipGetLastError();
}

hipError_t launch_eig_svd(const JacobiBlock* table_dev, const JacobiBlock* single, int blocks, int max_k,
                          hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    if (max_k > EIG_MAXK || max_k < 1) return hipErrorInvalidValue;
    JacobiBlock sb{};
    if (single) sb = *single;
    const int tiles = (max_k + 63) / 64;
    const EigGrid gt{blocks, tiles * tiles, 0};
    const EigGrid gv{blocks, (max_k + EIG_VAL_PER_WG - 1) / EIG_VAL_PER_WG, 0};
    const EigGrid gi{blocks, (max_k + 63) / 64, 1};      // measured: pinned 0.70 ms, chunk-major 0.74 (84 blocks, k = 264)
    hipLaunchKernelGGL(eig_gemm_kernel<0>, eig_grid(gt), dim3(256), 0, stream, table_dev, sb, gt);
    hipLaunchKernelGGL(eig_tridiag_kernel, dim3(blocks), dim3(EIG_THREADS), 0, stream, table_dev, sb);
    hipLaunchKernelGGL(eig_values_kernel, eig_grid(gv), dim3(256), 0, stream, table_dev, sb, gv);
    hipLaunchKernelGGL(eig_invit_kernel, eig_grid(gi), dim3(64), 0, stream, table_dev, sb, gi);
    hipLaunchKernelGGL(eig_groups_kernel, dim3(blocks), dim3(EIG_THREADS), 0, stream, table_dev, sb);
    const EigGrid gbt{blocks, tiles, 0};
    const dim3 bt_grid = eig_grid(gbt);
    if (max_k <= 32) hipLaunchKernelGGL((eig_backtransform_kernel<8, 4>), bt_grid, dim3(256), 0, stream, table_dev, sb, gbt);
    else if (max_k <= 96) hipLaunchKernelGGL((eig_backtransform_kernel<24, 4>), bt_grid, dim3(256), 0, stream, table_dev, sb, gbt);
    else if (max_k <= 160) hipLaunchKernelGGL((eig_backtransform_kernel<40, 4>), bt_grid, dim3(256), 0, stream, table_dev, sb, gbt);
    else if (max_k <= 320) hipLaunchKernelGGL((eig_backtransform_kernel<40, 8>), bt_grid, dim3(512), 0, stream, table_dev, sb, gbt);
    else hipLaunchKernelGGL((eig_backtransform_kernel<40, 16>), bt_grid, dim3(1024), 0, stream, table_dev, sb, gbt);
    hipLaunchKernelGGL(eig_gemm_kernel<1>, eig_grid(gt), dim3(256), 0, stream, table_dev, sb, gt);
    hipLaunchKernelGGL(eig_finish_kernel, dim3(blocks), dim3(EIG_THREADS), 0, stream, table_dev, sb);
    return hipGetLastError();
}

}  // namespace tsr
