// NG-SGD: online low-rank natural-gradient preconditioner (Sec. 4, eq. 4: theta <- theta + alpha E g with
// E symmetric positive definite, standing for the inverse Fisher matrix of eq. 5, approximated directly).
//
// State per preconditioned matrix (dimension D, rank R): R_t (R x D, orthonormal rows, float32), d_t (R),
// rho_t, t (float64 / int64); Fisher estimate F_t = R_t^T diag(d_t) R_t + rho_t I.
//   apply:  beta = rho(1+alpha) + alpha sum(d)/D;  e_i = d_i/(d_i+beta);  H = X R^T;  Xh = X - H diag(e) R;
//           out = Xh ||X||_F/||Xh||_F
//   fold:   Y = (eta/N) H^T X + (1-eta)(diag(d)+rho I) R;  Z = Y Y^T = U diag(c) U^T;  R' = diag(c)^-1/2 U^T Y;
//           rho' = [eta ||X||^2/N + (1-eta)(D rho + sum d) - sum sqrt c]/(D-R);  d' = sqrt(c) - rho';  floors.
// Xh is evaluated as  X1 = X - H R;  H2 = X1 R^T;  Xh = X1 + (H (I - E) - H2) R : the projection on the tracked
// subspace is taken out twice, because X often lies almost entirely inside it and a single float32 pass
// leaves the small remainder with a large relative error.
// The N x D and R x D work runs in float32 on the MFMA GEMM; the R x R work (Z, its Jacobi eigen-decomposition,
// d, rho) runs in float64 in one workgroup.  Every kernel takes a batch index (one state per replica).
// Every step of the apply is a kernel over a table of matrices (*_slots_kernel): ng_dnn_update takes all layer
// sides of a backward pass through each step in one launch, ng_run is the same recipe for a table of one.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "../../include/mavg.h"
#include "device_math.h"
#include "gemm.h"
#include "kernels.h"
#include "ng_internal.h"

namespace mavg {

namespace {

constexpr double kEps = 1e-10, kDelta = 5e-4, kCFloor = 1e-24;
constexpr int kInitFolds = 3;
constexpr int kMaxRank = 64;
constexpr int kJacobiSweeps = 14;
constexpr int kNgParts = 2048;     // partial sums of squares per (slot, replica)

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct StateView { float* R; double* d; double* rho; int64_t* t; int32_t* info; };
__host__ __device__ inline StateView state_view(char* st, int dim, int rank) {
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    StateView v;
    v.R = reinterpret_cast<float*>(st);
    v.d = reinterpret_cast<double*>(st + (int64_t)rank * ld * 4);
    v.rho = v.d + rank;
    v.t = reinterpret_cast<int64_t*>(v.rho + 1);
    v.info = reinterpret_cast<int32_t*>(v.t + 1);     // [0] Jacobi sweeps of the last fold, [1] folds that ran out of sweeps
    return v;
}

// The thin products H = X R^T run as one launch of 32-row tiles; to occupy the whole chip the contraction of each
// is cut into chunks of about 1024 (multiples of 16) whose partial products are summed afterwards.
inline int ng_chunk_len(int dim) {
    int nch = (dim + 512) / 1024;
    if (nch < 1) nch = 1;
    return (int)round_up((dim + nch - 1) / nch, 16);
}
inline int ng_chunk_count(int dim) { const int kc = ng_chunk_len(dim); return (dim + kc - 1) / kc; }

// scratch carve-up (offsets in floats from a 256-byte aligned base)
struct NgWs {
    int64_t ldr, ld;
    int64_t off_H, off_H2, H_b, off_Y, RY_b, off_coef, coef_b, off_gamma;
    int64_t off_scal, off_part, off_Z, off_Wt;       // float64 regions (offsets still in floats)
    int64_t off_H64, H64_b, off_Y64, Y64_b;          // float64 copies used by the initial folds
    int64_t off_P;                                   // partial products of the chunked thin GEMM
    int64_t off_gemm, gemm_floats, total;
};

NgWs ng_ws(int dim, int rank, int n, int batch) {
    NgWs w;
    w.ldr = round_up(rank, 4);
    w.ld = round_up(dim, 4);
    w.H_b = round_up((int64_t)n * w.ldr, 64);
    w.RY_b = round_up((int64_t)rank * w.ld, 64);
    w.coef_b = 3 * kMaxRank;
    w.gemm_floats = round_up(gemm_ws_floats(rank, dim, n, batch), 64);       // Y = H^T X
    int64_t off = 0;
    w.off_H = off;     off += w.H_b * batch;
    w.off_H2 = off;    off += w.H_b * batch;
    w.off_Y = off;     off += w.RY_b * batch;
    w.off_coef = off;  off += w.coef_b * batch;
    w.off_gamma = off; off += round_up(2 * (int64_t)batch, 64);
    w.off_scal = off;  off += round_up(2 * 2 * (int64_t)batch, 64);
    w.off_part = off;  off += 2 * kNgParts * (int64_t)batch;
    w.off_Z = off;     off += 2 * (int64_t)kMaxRank * kMaxRank * batch;
    w.off_Wt = off;    off += 2 * (int64_t)kMaxRank * kMaxRank * batch;
    w.H64_b = 2 * (int64_t)n * kMaxRank;
    w.Y64_b = 2 * round_up((int64_t)rank * w.ld, 64);
    w.off_H64 = off;   off += w.H64_b * batch;
    w.off_Y64 = off;   off += w.Y64_b * batch;
    w.off_P = off;     off += (int64_t)ng_chunk_count(dim) * batch * w.H_b;
    w.off_gemm = off;  off += w.gemm_floats;
    w.total = off;
    return w;
}

__device__ __forceinline__ double block_sum_d(double v, double* sh) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const double r = (sh[0] + sh[1]) + (sh[2] + sh[3]);
    __syncthreads();
    return r;
}

// the eigen-solver runs 512 threads: 16 groups of 32 lanes, one group per rotation pair up to rank 32
constexpr int kEigThreads = 512;
constexpr int kEigSoloLds = 120 * 1024;      // bytes of LDS a solver workgroup asks for to have its compute unit to itself
constexpr int kEigSoloMax = 64;              // ... in launches of at most this many workgroups
__device__ __forceinline__ double block_sum_eig(double v, double* sh) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    const double r = ((sh[0] + sh[1]) + (sh[2] + sh[3])) + ((sh[4] + sh[5]) + (sh[6] + sh[7]));
    __syncthreads();
    return r;
}

// Table of independent folds finished by one launch of each of ng_z_kernel / ng_eig_kernel / ng_newr_kernel:
// slot = one preconditioned matrix (a layer's input or output side), times `batch` replicas.
constexpr int kNgSlots = 32;
struct NgFoldTable {
    char* state[kNgSlots];          // state of (slot, replica 0); replica b at + b * st_b bytes
    const void* Y[kNgSlots];        // Y of (slot, replica 0), float or double; replica b at + b * y_b[slot] elements
    int64_t y_b[kNgSlots];
    const double* scal[kNgSlots];   // [batch][2]: ||X||^2, ||Xh||^2
    int dim[kNgSlots];
    int64_t st_b;
    int nslots, batch, first;       // first: index of slot 0 in the Z / Wt scratch arrays
};

// ---- kernels -------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void ng_init_kernel(char* state, int dim, int rank) {
    const StateView v = state_view(state, dim, rank);
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < (int64_t)rank * ld; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / ld, c = i - r * ld;
        v.R[i] = (r == c) ? 1.f : 0.f;
    }
    if (blockIdx.x == 0) {
        if (threadIdx.x < rank) v.d[threadIdx.x] = kEps;
        if (threadIdx.x == 0) { *v.rho = kEps; *v.t = 0; v.info[0] = 0; v.info[1] = 0; }
    }
}

__global__ __launch_bounds__(256) void ng_scale_kernel(float* __restrict__ x, int64_t ldx, int64_t x_b, int n, int dim,
                                                       const float* __restrict__ gamma) {
    const int b = blockIdx.y;
    const float g = gamma[b];
    const int64_t total = (int64_t)n * dim;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
        const int64_t r = e / dim, c = e - r * dim;
        x[(int64_t)b * x_b + r * ldx + c] *= g;
    }
}

// Z = Y Y^T in float64; one workgroup per (i <= j)
template <typename YT>
__global__ __launch_bounds__(256) void ng_z_kernel(NgFoldTable tb, int rank, double* __restrict__ Z) {
    __shared__ double sh[4];
    const int slot = blockIdx.y, b = blockIdx.z;
    const int i = blockIdx.x / rank, j = blockIdx.x - i * rank;
    if (i > j) return;
    const int dim = tb.dim[slot];
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    const YT* __restrict__ Y = static_cast<const YT*>(tb.Y[slot]) + (int64_t)b * tb.y_b[slot];
    const YT* __restrict__ yi = Y + (int64_t)i * ld;
    const YT* __restrict__ yj = Y + (int64_t)j * ld;
    double s = 0.0;
    for (int c = threadIdx.x; c < dim; c += 256) s += (double)yi[c] * (double)yj[c];
    s = block_sum_d(s, sh);
    if (threadIdx.x == 0) {
        double* Zb = Z + ((int64_t)(tb.first + slot) * tb.batch + b) * kMaxRank * kMaxRank;
        Zb[i * rank + j] = s;
        Zb[j * rank + i] = s;
    }
}

// Reciprocal square root and reciprocal in float64 from the hardware's approximations and two Newton steps each
// (relative error at rounding level for normal arguments; no special-case handling: the callers pass positive, finite,
// normal values).
__device__ __forceinline__ double fast_rsqrt(double x) {
    double y = __builtin_amdgcn_rsq(x);
    y = y * (1.5 - 0.5 * x * y * y);
    y = y * (1.5 - 0.5 * x * y * y);
    return y;
}
__device__ __forceinline__ double fast_rcp(double x) {
    double y = __builtin_amdgcn_rcp(x);
    y = y * (2.0 - x * y);
    y = y * (2.0 - x * y);
    return y;
}

// Symmetric eigen-decomposition of the rank x rank matrix Z by cyclic Jacobi rotations in a round-robin
// (tournament) order, so that the rank/2 disjoint rotations of a round are applied in parallel, rows and
// columns in one pass (the column partner's entries come from a neighbouring lane); then the
// new d, rho, t and the matrix Wt = diag(c)^-1/2 U^T (rows in descending order of c).
//
// Threads form groups of 32 lanes (64 above rank 32), lane l standing for index l of the matrix.  In round `rd` of
// the tournament among m = rank rounded up to even players, player m-1 meets player rd and every other player l
// meets (2 rd - l) mod (m - 1); an odd rank leaves the player that would meet the dummy idle.  Every lane works out
// the rotation of its own index's pair from the three entries it depends on (all groups do so redundantly: no
// hand-over through LDS, no barrier between computing the rotations and applying them); the group that owns a pair's
// two rows takes that pair's rotation from its lane p.  Z and U^T are kept twice: a round reads one copy and writes the
// other (every row belongs to exactly one pair, or is the idle one, and is written once per round), so a wavefront
// that is ahead never overwrites what a slower one still has to read, and one barrier per round is enough.
__global__ __launch_bounds__(kEigThreads) void ng_eig_kernel(NgFoldTable tb, int rank, int n, float eta, const double* __restrict__ Zg,
                                                     double* __restrict__ Wt, int bump_t) {
    extern __shared__ double smem[];
    const int r = rank;
    const int rs = (r + 1) & ~1;     // even row stride: the diagonal (stride rs + 1 doubles, odd) spreads over all LDS banks
    double* Zs = smem;               // r x rs, current copy (the two copies swap after every round)
    double* Us = Zs + r * rs;        // r x rs, holds U TRANSPOSED (row k = eigenvector k), so its update is a row rotation
    double* Zn = Us + r * rs;        // the copies the current round writes
    double* Un = Zn + r * rs;
    double* red = Un + r * rs;       // 16
    int* order = reinterpret_cast<int*>(red + 16);   // 64
    const int slot = blockIdx.x / tb.batch, b = blockIdx.x - slot * tb.batch, tid = threadIdx.x;
    const int dim = tb.dim[slot];
    const int64_t zi = (int64_t)(tb.first + slot) * tb.batch + b;
    const double* __restrict__ Zb = Zg + zi * kMaxRank * kMaxRank;
    // thread = (lane: an index along a row, grp: which rotation pair / which row); a group never straddles a wavefront
    const int lw = r <= 32 ? 32 : 64, ngrp = kEigThreads / lw;
    const int lane = tid & (lw - 1), grp = tid / lw;
    for (int i = grp; i < r; i += ngrp)
        if (lane < r) {
            Zs[i * rs + lane] = Zb[i * r + lane];
            Us[i * rs + lane] = (i == lane) ? 1.0 : 0.0;
        }
    __syncthreads();
    const int m = (r + 1) & ~1;      // even number of players
    const int half = m / 2;
    const bool on = lane < r;
    int sweeps_done = 0;
    bool converged = false;
    for (int sweep = 0; sweep <= kJacobiSweeps; ++sweep) {
        // stop when the off-diagonal mass is negligible against the diagonal
        double off = 0.0, dg = 0.0;
        for (int i = grp; i < r; i += ngrp)
            if (on) {
                const double v = Zs[i * rs + lane];
                if (i == lane) dg += v * v; else off += v * v;
            }
        off = wave_sum(off);
        dg = wave_sum(dg);
        if ((tid & 63) == 0) { red[tid >> 6] = off; red[8 + (tid >> 6)] = dg; }
        __syncthreads();
        off = ((red[0] + red[1]) + (red[2] + red[3])) + ((red[4] + red[5]) + (red[6] + red[7]));
        dg = ((red[8] + red[9]) + (red[10] + red[11])) + ((red[12] + red[13]) + (red[14] + red[15]));
        __syncthreads();
        // off-diagonal norm below 1e-13 of the diagonal: Z spans many orders of magnitude, and a looser stop (1e-10)
        // leaves its small eigenvalues, hence the weak rows of R, outside the parity tolerance
        if (off <= 1e-26 * dg) { converged = true; break; }
        if (sweep == kJacobiSweeps) break;          // out of sweeps: the state's info word counts it
        ++sweeps_done;
        for (int round = 0; round < m - 1; ++round) {
            // Z <- J^T Z J, U^T <- J^T U^T with, for every pair (p, q), p < q, of the round,
            // row_p <- c row_p - s row_q,  row_q <- s row_p + c row_q  (and the same for the columns of Z)
            int pl = lane;                               // the index this lane's index meets (itself: idle)
            if (on) {
                int w = 2 * round - lane;                // in (-(m-1), 2(m-1)): reduce mod m-1 without a division
                if (w < 0) w += m - 1;
                if (w >= m - 1) w -= m - 1;
                pl = lane == m - 1 ? round : lane == round ? m - 1 : w;
                if (pl >= r) pl = lane;                  // the bye of an odd rank
            }
            double cl = 1.0, sl = 0.0;                   // rotation of the pair this lane's index is in
            if (pl != lane) {
                const int p = min(lane, pl), q = max(lane, pl);
                const double app = Zs[p * rs + p], aqq = Zs[q * rs + q], apq = Zs[p * rs + q];
                // t = sgn(tau) / (|tau| + sqrt(1 + tau^2)) with tau = (aqq - app) / (2 apq)
                const double d = aqq - app, b2 = 2.0 * apq;
                const double h2 = d * d + b2 * b2;
                if (apq != 0.0 && h2 > 1e-280) {         // (below that the entry is nothing against any diagonal)
                    const double t = (d >= 0.0 ? b2 : -b2) * fast_rcp(fabs(d) + h2 * fast_rsqrt(h2));
                    cl = fast_rsqrt(1.0 + t * t);
                    sl = t * cl;
                }
            }
            // row `lane` (and column `lane`) turns into al row_lane + bl row_partner
            const double al = cl, bl = lane < pl ? -sl : sl;
            // One pass: the group of pair k holds rows p and q; lane l rotates the rows (in registers), fetches the
            // rotated entries of column partner(l) from the lane that holds them and rotates the columns.
            for (int k = grp; k < half; k += ngrp) {
                int p, q;
                if (k == 0) { p = m - 1; q = round; }
                else {
                    p = round + k;     if (p >= m - 1) p -= m - 1;
                    q = round - k;     if (q < 0) q += m - 1;
                }
                if (p > q) { const int t = p; p = q; q = t; }
                const bool two = q < r;                  // else the bye: row and column p stay
                const int qr = two ? q : p;
                const double c = two ? __shfl(cl, p, lw) : 1.0, s = two ? __shfl(sl, p, lw) : 0.0;
                const double zp = on ? Zs[p * rs + lane] : 0.0, zq = (on && two) ? Zs[qr * rs + lane] : 0.0;
                const double up = on ? Us[p * rs + lane] : 0.0, uq = (on && two) ? Us[qr * rs + lane] : 0.0;
                const double wp = c * zp - s * zq, wq = s * zp + c * zq;
                const double wpo = __shfl(wp, pl, lw), wqo = __shfl(wq, pl, lw);
                if (on) {
                    Zn[p * rs + lane] = al * wp + bl * wpo;
                    Un[p * rs + lane] = c * up - s * uq;
                    if (two) {
                        Zn[q * rs + lane] = al * wq + bl * wqo;
                        Un[q * rs + lane] = s * up + c * uq;
                    }
                }
            }
            __syncthreads();
            { double* t = Zs; Zs = Zn; Zn = t; t = Us; Us = Un; Un = t; }
        }
    }
    // descending order of the eigenvalues (ties by index)
    if (tid < r) {
        const double ci = Zs[tid * rs + tid];
        int pos = 0;
        for (int j = 0; j < r; ++j) {
            const double cj = Zs[j * rs + j];
            if (cj > ci || (cj == ci && j < tid)) ++pos;
        }
        order[pos] = tid;
    }
    __syncthreads();
    const StateView v = state_view(tb.state[slot] + (int64_t)b * tb.st_b, dim, rank);
    if (tid == 0) {
        const double cmax = Zs[order[0] * rs + order[0]];
        double sumd = 0.0, sumsq = 0.0;
        for (int j = 0; j < r; ++j) sumd += v.d[j];
        const double rho = *v.rho;
        for (int i = 0; i < r; ++i) {
            double c = Zs[order[i] * rs + order[i]];
            c = fmax(c, kCFloor * cmax);
            const double sq = sqrt(c);
            Zs[order[i] * rs + order[i]] = sq;          // keep sqrt(c_i) on the diagonal for the other threads
            sumsq += sq;
        }
        const double trT = (double)eta * tb.scal[slot][b * 2 + 0] / (double)n + (1.0 - (double)eta) * ((double)dim * rho + sumd);
        double rho_new = (trT - sumsq) / (double)(dim - rank);
        double dmax = -1e300;
        for (int i = 0; i < r; ++i) {
            const double di = Zs[order[i] * rs + order[i]] - rho_new;
            v.d[i] = di;
            dmax = fmax(dmax, di);
        }
        rho_new = fmax(rho_new, kEps);
        const double floor_d = fmax(kEps, kDelta * dmax);
        for (int i = 0; i < r; ++i) v.d[i] = fmax(v.d[i], floor_d);
        *v.rho = rho_new;
        if (bump_t) *v.t = *v.t + 1;
        v.info[0] = sweeps_done;
        if (!converged) v.info[1] += 1;
    }
    __syncthreads();
    double* __restrict__ Wb = Wt + zi * kMaxRank * kMaxRank;
    for (int w = tid; w < r * r; w += kEigThreads) {
        const int i = w / r, k = w - i * r;
        const int col = order[i];
        Wb[w] = Us[col * rs + k] / Zs[col * rs + col];
    }
}

// R' = Wt Y (float64 accumulation).  A workgroup owns 32 columns; its 8 thread rows each produce every 8th row of R'.
template <typename YT>
__global__ __launch_bounds__(256) void ng_newr_kernel(NgFoldTable tb, int rank, const double* __restrict__ Wt) {
    __shared__ double Ws[kMaxRank * kMaxRank];
    __shared__ YT ys[kMaxRank][33];
    const int slot = blockIdx.y, b = blockIdx.z;
    const int dim = tb.dim[slot];
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    if ((int64_t)blockIdx.x * 32 >= ld) return;
    const double* __restrict__ Wb = Wt + ((int64_t)(tb.first + slot) * tb.batch + b) * kMaxRank * kMaxRank;
    for (int i = threadIdx.x; i < rank * rank; i += 256) Ws[i] = Wb[i];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + tx;
    const YT* __restrict__ Yb = static_cast<const YT*>(tb.Y[slot]) + (int64_t)b * tb.y_b[slot];
    for (int k = ty; k < rank; k += 8) ys[k][tx] = (c < dim) ? Yb[(int64_t)k * ld + c] : (YT)0;
    __syncthreads();
    if (c >= ld) return;
    float* __restrict__ R = state_view(tb.state[slot] + (int64_t)b * tb.st_b, dim, rank).R;
    for (int i = ty; i < rank; i += 8) {
        double acc = 0.0;
        for (int k = 0; k < rank; ++k) acc += Ws[i * rank + k] * (double)ys[k][tx];
        R[(int64_t)i * ld + c] = (c < dim) ? (float)acc : 0.f;
    }
}

// Float64 versions of H = X R^T and Y = (eta/n) H^T X + (1-eta)(diag(d)+rho I) R for the folds that start from the
// initial state: there the rows of Y are all dominated by the leading direction of the data and the weaker
// directions sit below float32 resolution.
__global__ __launch_bounds__(256) void ng_h64_kernel(char* state, int64_t st_b, int dim, int rank, const float* __restrict__ x,
                                                     int64_t ldx, int64_t x_b, double* __restrict__ H64, int64_t h_b) {
    __shared__ double sh[4];
    const int b = blockIdx.y, r = blockIdx.x;
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    const float* __restrict__ R = state_view(state + (int64_t)b * st_b, dim, rank).R;
    const float* __restrict__ row = x + (int64_t)b * x_b + (int64_t)r * ldx;
    double acc[kMaxRank];
#pragma unroll
    for (int i = 0; i < kMaxRank; ++i) acc[i] = 0.0;
    for (int c = threadIdx.x; c < dim; c += 256) {
        const double xv = (double)row[c];
#pragma unroll
        for (int i = 0; i < kMaxRank; ++i)
            if (i < rank) acc[i] += xv * (double)R[(int64_t)i * ld + c];
    }
    double* __restrict__ out = H64 + ((int64_t)b * h_b) / 2 + (int64_t)r * kMaxRank;
#pragma unroll
    for (int i = 0; i < kMaxRank; ++i) {
        if (i < rank) {                       // uniform across the workgroup
            const double v = block_sum_d(acc[i], sh);
            if (threadIdx.x == 0) out[i] = v;
        }
    }
}

__global__ __launch_bounds__(256) void ng_y64_kernel(char* state, int64_t st_b, int dim, int rank, int n, float eta,
                                                     const float* __restrict__ x, int64_t ldx, int64_t x_b,
                                                     const double* __restrict__ H64, int64_t h_b, double* __restrict__ Y64, int64_t y_b) {
    __shared__ double hs[16][kMaxRank];
    const int b = blockIdx.y;
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    const StateView v = state_view(state + (int64_t)b * st_b, dim, rank);
    const int c = blockIdx.x * 256 + threadIdx.x;
    const float* __restrict__ xb = x + (int64_t)b * x_b;
    const double* __restrict__ Hb = H64 + ((int64_t)b * h_b) / 2;
    double acc[kMaxRank];
#pragma unroll
    for (int i = 0; i < kMaxRank; ++i) acc[i] = 0.0;
    for (int n0 = 0; n0 < n; n0 += 16) {
        __syncthreads();
        for (int w = threadIdx.x; w < 16 * kMaxRank; w += 256) {
            const int rr = w / kMaxRank, i = w - rr * kMaxRank;
            hs[rr][i] = (n0 + rr < n && i < rank) ? Hb[(int64_t)(n0 + rr) * kMaxRank + i] : 0.0;
        }
        __syncthreads();
        if (c < dim) {
            for (int rr = 0; rr < 16 && n0 + rr < n; ++rr) {
                const double xv = (double)xb[(int64_t)(n0 + rr) * ldx + c];
#pragma unroll
                for (int i = 0; i < kMaxRank; ++i)
                    if (i < rank) acc[i] += hs[rr][i] * xv;
            }
        }
    }
    if (c < dim) {
        const double rho = *v.rho, s = (double)eta / (double)n;
        double* __restrict__ Yb = Y64 + ((int64_t)b * y_b) / 2;
#pragma unroll
        for (int i = 0; i < kMaxRank; ++i)
            if (i < rank) Yb[(int64_t)i * ld + c] = s * acc[i] + (1.0 - (double)eta) * (v.d[i] + rho) * (double)v.R[(int64_t)i * ld + c];
    }
}


// ---- the steps of the apply, for a table of matrices ------------------------------------------------
//
// Between the end of the back-propagation chain and the weight updates the 2 L preconditioned matrices of a
// network (input and output side of every layer) are independent of each other.  One preconditioning is a dozen
// small launches, each a few microseconds of mostly latency; the kernels below take a table of slots (one slot =
// one matrix, times `batch` replicas) so that a whole backward pass needs one launch per step of the recipe
// instead of one per step and matrix.  A single matrix (ngsgd_precondition, the first minibatch of a network) is
// a table of one slot.
struct NgSlots {
    char* state[kNgSlots];          // state of (slot, replica 0); replica b at + b * st_b bytes
    float* x[kNgSlots];             // matrix of (slot, replica 0), n x dim, preconditioned in place
    int64_t ldx[kNgSlots], x_b[kNgSlots];
    int dim[kNgSlots];
    int64_t st_b;
    int nslots, batch, n, rank;
    // scratch with one stride per (slot, replica) pair q = slot * batch + b
    float* H; float* H2; int64_t ldr, H_b;      // n x ldr each, at + q * H_b
    float* coef;                                // at + q * 3 kMaxRank
    double* part;                               // at + q * kNgParts
    double* scal;                               // at + q * 2: ||X||^2, ||Xh||^2
    float* gamma;                               // at + q
    float* wcol = nullptr;                      // optional, at + q * n: receives the last column of the preconditioned matrix
};

__global__ __launch_bounds__(256) void ng_sumsq_partial_slots_kernel(NgSlots t, int write_lastcol) {
    __shared__ double sh[4];
    const int slot = blockIdx.y, b = blockIdx.z;
    const int64_t q = (int64_t)slot * t.batch + b;
    const float* __restrict__ xb = t.x[slot] + (int64_t)b * t.x_b[slot];
    const int64_t ldx = t.ldx[slot];
    const int dim = t.dim[slot], n = t.n;
    const bool vec = (ldx & 3) == 0 && (t.x_b[slot] & 3) == 0 && (reinterpret_cast<uintptr_t>(t.x[slot]) & 15u) == 0;
    double s = 0.0;
    for (int r = blockIdx.x; r < n; r += gridDim.x) {
        const float* __restrict__ row = xb + (int64_t)r * ldx;
        if (write_lastcol && threadIdx.x == 0) t.wcol[q * n + r] = row[dim - 1];
        float a = 0.f;
        if (vec) {
            const int nq = dim >> 2;
            int c4 = threadIdx.x;
            for (; c4 + 768 < nq; c4 += 1024) {
                const float4 v0 = *reinterpret_cast<const float4*>(row + 4 * c4);
                const float4 v1 = *reinterpret_cast<const float4*>(row + 4 * (c4 + 256));
                const float4 v2 = *reinterpret_cast<const float4*>(row + 4 * (c4 + 512));
                const float4 v3 = *reinterpret_cast<const float4*>(row + 4 * (c4 + 768));
                a += (v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w);
                a += (v1.x * v1.x + v1.y * v1.y) + (v1.z * v1.z + v1.w * v1.w);
                a += (v2.x * v2.x + v2.y * v2.y) + (v2.z * v2.z + v2.w * v2.w);
                a += (v3.x * v3.x + v3.y * v3.y) + (v3.z * v3.z + v3.w * v3.w);
            }
            for (; c4 < nq; c4 += 256) {
                const float4 v0 = *reinterpret_cast<const float4*>(row + 4 * c4);
                a += (v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w);
            }
            for (int c = 4 * nq + threadIdx.x; c < dim; c += 256) { const float e = row[c]; a += e * e; }
        } else {
            for (int c = threadIdx.x; c < dim; c += 256) { const float e = row[c]; a += e * e; }
        }
        s += (double)a;
    }
    s = block_sum_d(s, sh);
    if (threadIdx.x == 0) t.part[q * kNgParts + blockIdx.x] = s;
}

// The coefficients of the apply and the fold of (slot, replica b) from its state: e, (1 - eta)(d + rho), 1 - e.
// By the first `rank` threads of a workgroup.
__device__ __forceinline__ void ng_coefficients(const NgSlots& t, int slot, int b, float alpha, float eta) {
    const int64_t q = (int64_t)slot * t.batch + b;
    const int dim = t.dim[slot], rank = t.rank;
    const StateView v = state_view(t.state[slot] + (int64_t)b * t.st_b, dim, rank);
    double sumd = 0.0;
    for (int j = 0; j < rank; ++j) sumd += v.d[j];
    const double rho = *v.rho;
    const double beta = rho * (1.0 + (double)alpha) + (double)alpha * sumd / (double)dim;
    if ((int)threadIdx.x < rank) {
        const double di = v.d[threadIdx.x];
        float* __restrict__ cf = t.coef + q * (3 * kMaxRank);
        cf[threadIdx.x] = (float)(di / (di + beta));
        cf[kMaxRank + threadIdx.x] = (float)((1.0 - (double)eta) * (di + rho));
        cf[2 * kMaxRank + threadIdx.x] = (float)(beta / (di + beta));
    }
}

// what & 1: sum the first `nparts` partial sums of every (slot, replica) in index order into scal[q][which]
//           (which 0: ||X||^2, which 1: ||Xh||^2 and gamma[q] = ||X|| / ||Xh||, 1 if either is 0);
// what & 2: the coefficients of the apply and the fold from the state (e, (1 - eta)(d + rho), 1 - e)
__global__ __launch_bounds__(256) void ng_sumsq_final_slots_kernel(NgSlots t, int which, float alpha, float eta, int nparts, int what) {
    __shared__ double sh[4];
    const int slot = blockIdx.x, b = blockIdx.y;
    const int64_t q = (int64_t)slot * t.batch + b;
    if (what & 1) {
        double s = 0.0;
        for (int i = threadIdx.x; i < nparts; i += 256) s += t.part[q * kNgParts + i];
        s = block_sum_d(s, sh);
        if (threadIdx.x == 0) {
            t.scal[q * 2 + which] = s;
            if (which == 1) {
                const double nx = t.scal[q * 2 + 0];
                t.gamma[q] = (nx > 0.0 && s > 0.0) ? (float)sqrt(nx / s) : 1.f;
            }
        }
    }
    if (what & 2) ng_coefficients(t, slot, b, alpha, eta);
}

// Hout of every slot = sum of the slot's partial products (one per chunk of the contraction), in chunk order
struct NgChunkTable { int first[kNgSlots], count[kNgSlots]; };
// combine != 0 (Hout = t.H2): what is left is H (I - E) - (that sum) in the columns below the rank, the combination
// the second rank update multiplies by R
__global__ __launch_bounds__(256) void ng_sum_chunks_slots_kernel(NgSlots t, NgChunkTable ct, const float* __restrict__ P,
                                                                  float* __restrict__ Hout, int combine) {
    const int slot = blockIdx.y, b = blockIdx.z;
    const int64_t q = (int64_t)slot * t.batch + b;
    const int64_t total4 = (int64_t)t.n * t.ldr / 4;            // ldr is a multiple of 4
    const int first = ct.first[slot], count = ct.count[slot];
    float4* __restrict__ out = reinterpret_cast<float4*>(Hout + q * t.H_b);
    const float* __restrict__ ome = t.coef + q * (3 * kMaxRank) + 2 * kMaxRank;
    const float4* __restrict__ H4 = reinterpret_cast<const float4*>(t.H + q * t.H_b);
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total4; e += (int64_t)gridDim.x * 256) {
        float4 a = reinterpret_cast<const float4*>(P + ((int64_t)first * t.batch + b) * t.H_b)[e];
        for (int c = 1; c < count; ++c) {
            const float4 v = reinterpret_cast<const float4*>(P + ((int64_t)(first + c) * t.batch + b) * t.H_b)[e];
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        if (combine) {
            const int i = (int)((4 * e) % t.ldr);               // column of a.x; the four elements share a row
            const float4 h = H4[e];
            if (i + 0 < t.rank) a.x = h.x * ome[i + 0] - a.x;
            if (i + 1 < t.rank) a.y = h.y * ome[i + 1] - a.y;
            if (i + 2 < t.rank) a.z = h.z * ome[i + 2] - a.z;
            if (i + 3 < t.rank) a.w = h.w * ome[i + 3] - a.w;
        }
        out[e] = a;
    }
}

// X <- X + sign * Cm R for every slot (Cm = H or H2 of the slot) on the matrix cores: a wavefront owns 32
// columns, keeps its 32 (x KH) x 32 block of R in registers as MFMA B operands and walks down `rows` rows in tiles
// of 32; per tile it reads 32 x rank of Cm (16 contiguous floats per lane) and 32 x 32 of X, multiplies with
// 16 KH v_mfma_f32_32x32x2_f32 and adds the product to X.  Contraction index of MFMA step s: k = 32 kh + s in
// lanes 0-31 and 32 kh + 16 + s in lanes 32-63, zero operands beyond `rank`.  No LDS in the loop, no barrier.
// (The other order - the block of Cm in registers, walking along the columns and reading a block of R per 32 x 32 of
// X - was measured slower, 56 against 42 us for the 14 matrices of 512 rows of the 440-6x2048-8000 network: the blocks of R,
// 3.4 MB in all, do not stay in the L2 beside the stream of X.)
//
// `fuse` folds the passes over the matrices that take the norms into the two rank updates of a preconditioning:
//   0  nothing else;
//   1  (first update, X1 = X - H R) also leaves the workgroup's share of ||X||^2, of X as it was read;
//   2  (second update) also leaves the workgroup's share of ||Xh||^2 of the result, and the result's last column in
//      t.wcol.
// The shares go to t.part[q][blockIdx.y * maxblk + (block of 128 columns)]; a slot's last workgroup of a row zeroes the
// entries up to maxblk, so that every slot has the same number of shares to sum.
// (Summing the chunks of H2 and forming H (I - E) - H2 on the way in as well was measured slower: every one of the
// up to 250 column blocks of a slot would redo that sum.)
typedef float ng_floatx16 __attribute__((ext_vector_type(16)));
// A pointer that is uniform over the wavefront, pinned to scalar registers: an access through it plus a 32-bit
// per-lane offset takes the scalar-base form of the memory instructions, one offset register per access pattern
// instead of a 64-bit address per access.  (The result is typed as a pointer to global memory: rebuilt from an
// integer, a plain pointer would be accessed with flat instructions.)
typedef __attribute__((address_space(1))) char ng_gchar;
typedef __attribute__((address_space(1))) float ng_gfloat;
__device__ __forceinline__ ng_gchar* ng_uniform_ptr(const char* p) {
    const uint64_t x = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return reinterpret_cast<ng_gchar*>(((uint64_t)hi << 32) | lo);
}
// Where Y of every slot goes (replica b at + b * y_b floats), and, for the rank update that takes Y's product with
// it, where the partial products go: that of the rows of workgroup row c at P + c * p_chunk (+ b * y_b), laid out like Y.
struct NgYTable { float* Y[kNgSlots]; int64_t y_b[kNgSlots]; float* P[kNgSlots]; int64_t p_chunk; };
// WITHY (with fuse 1, Cm = H): the launch also leaves H^T X of its rows, X as it was read, for the fold of the
// state (Y = alpha H^T X + diag(coef1) R, finished by ng_y_reduce_slots_kernel): X's block is in registers in the
// layout of an MFMA B operand already (lane = column; MFMA step v multiplies row 8 (v / 4) + v % 4 in lanes 0-31 and
// the row four further on in lanes 32-63), so the product costs 16 KH loads of H from the caches and 16 KH MFMAs
// per block instead of a pass of its own over X.
// The launch's x dimension runs through the blocks of 128 columns of all slots, one slot after the other (slot j:
// start[j] .. start[j + 1] - 1; a grid as wide as the widest slot for every slot had 70 % of its workgroups find
// nothing to do on the 440-6x2048-8000 network, and they cost a third of the launch); maxblk = the widest slot's count.
struct NgRuGrid { int start[kNgSlots + 1]; int maxblk; };
template <int KH, int FUSE, bool WITHY>
__global__ __launch_bounds__(256) void ng_rank_update_slots_kernel(NgSlots t, int use_h2, float sign, int rows, NgYTable yt, NgRuGrid g) {
    constexpr int fuse = FUSE;
    __shared__ double sh[4];
    int slot = 0;
#pragma unroll
    for (int j = 1; j < kNgSlots; ++j)
        if (j < t.nslots && (int)blockIdx.x >= g.start[j]) slot = j;
    slot = __builtin_amdgcn_readfirstlane(slot);
    const int xb = (int)blockIdx.x - g.start[slot], nblk = g.start[slot + 1] - g.start[slot], b = blockIdx.z;
    const int dim = t.dim[slot], n = t.n, rank = t.rank;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, h = lane >> 5, lc = lane & 31;
    const int c0 = (xb * 4 + wave) * 32;                // (uniform over the wavefront)
    const int64_t q = (int64_t)slot * t.batch + b;
    float ssq = 0.f;
    if (c0 < dim) {                                     // (the last block of a slot may have fewer than four wavefronts' worth)
        const int col = c0 + lc;
        const bool col_ok = col < dim;
        const int lcc = min(lc, dim - 1 - c0);          // the lane's column of the block, clamped for the loads
        const int64_t ldR = ((int64_t)dim + 3) / 4 * 4, ldx = t.ldx[slot], ldc = t.ldr;
        const uint32_t ldx4 = (uint32_t)ldx * 4u, ldR4 = (uint32_t)ldR * 4u;       // bytes per row
        const char* __restrict__ Rc = reinterpret_cast<const char*>(t.state[slot] + (int64_t)b * t.st_b) + (int64_t)c0 * 4;
        const float* __restrict__ C = (use_h2 ? t.H2 : t.H) + q * t.H_b;
        float* __restrict__ X = t.x[slot] + (int64_t)b * t.x_b[slot];
        // the block of R: (uniform) row min(ku, rank - 1); a lane whose own row ku + 16 lies beyond R reads that row instead
        const uint32_t offR0 = (uint32_t)lcc * 4u, offR1 = offR0 + (uint32_t)(16 * h) * ldR4;
        float bf[KH][16];
#pragma unroll
        for (int kh = 0; kh < KH; ++kh)
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const int ku = min(32 * kh + s, rank - 1);
                const ng_gchar* rowp = ng_uniform_ptr(Rc + (uint32_t)ku * ldR4);
                bf[kh][s] = *reinterpret_cast<const ng_gfloat*>(rowp + (32 * kh + s + 16 < rank ? offR1 : offR0));
            }
#pragma unroll
        for (int kh = 0; kh < KH; ++kh)
#pragma unroll
            for (int s = 0; s < 16; ++s)
                if (!(32 * kh + 16 * h + s < rank && col_ok)) bf[kh][s] = 0.f;
        const uint32_t offX = (uint32_t)lcc * 4u + (uint32_t)(4 * h) * ldx4;
        const int rbeg = blockIdx.y * rows, rend = min(n, rbeg + rows);
        const uint32_t ldc4 = (uint32_t)ldc * 4u;
        uint32_t offHy[KH];
        ng_floatx16 yacc[KH];
#pragma unroll
        for (int kh = 0; kh < KH; ++kh) {
            offHy[kh] = (uint32_t)min(32 * kh + lc, (int)ldc - 1) * 4u + (uint32_t)(4 * h) * ldc4;
            yacc[kh] = ng_floatx16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        }
        for (int r0 = rbeg; r0 < rend; r0 += 32) {
            const int row = r0 + lc;
            const bool interior = r0 + 32 <= rend;      // (uniform) else per-lane addresses and row checks
            const char* Xr = reinterpret_cast<const char*>(X + (int64_t)r0 * ldx) + (int64_t)c0 * 4;
            float af[KH][16];
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k4 = 32 * kh + 16 * h + 4 * j;
                    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (row < rend && k4 < ldc) v = *reinterpret_cast<const float4*>(C + (int64_t)row * ldc + k4);   // ldc is a multiple of 4
                    af[kh][4 * j + 0] = (k4 + 0 < rank) ? v.x : 0.f;
                    af[kh][4 * j + 1] = (k4 + 1 < rank) ? v.y : 0.f;
                    af[kh][4 * j + 2] = (k4 + 2 < rank) ? v.z : 0.f;
                    af[kh][4 * j + 3] = (k4 + 3 < rank) ? v.w : 0.f;
                }
            float old[16];
            if (interior) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    old[v] = *reinterpret_cast<const ng_gfloat*>(ng_uniform_ptr(Xr + (uint32_t)(8 * (v >> 2) + (v & 3)) * ldx4) + offX);
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (!col_ok) old[v] = 0.f;
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rr = r0 + 8 * (v >> 2) + 4 * h + (v & 3);
                    old[v] = (rr < rend && col_ok) ? X[(int64_t)rr * ldx + col] : 0.f;
                }
            }
            if (fuse == 1) {
#pragma unroll
                for (int v = 0; v < 16; ++v) ssq += old[v] * old[v];
            }
            if constexpr (WITHY) {       // H^T X of this block of rows: lane i of the A operand holds H(row of the step, i)
                float hy[KH][16];
                if (interior) {
                    const char* Hr = reinterpret_cast<const char*>(C + (int64_t)r0 * ldc);
#pragma unroll
                    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            hy[kh][v] = *reinterpret_cast<const ng_gfloat*>(ng_uniform_ptr(Hr + (uint32_t)(8 * (v >> 2) + (v & 3)) * ldc4) + offHy[kh]);
                } else {
#pragma unroll
                    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int rr = r0 + 8 * (v >> 2) + 4 * h + (v & 3);
                            hy[kh][v] = (rr < rend && 32 * kh + lc < rank) ? C[(int64_t)rr * ldc + 32 * kh + lc] : 0.f;
                        }
                }
#pragma unroll
                for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                    for (int v = 0; v < 16; ++v) yacc[kh] = __builtin_amdgcn_mfma_f32_32x32x2f32(hy[kh][v], old[v], yacc[kh], 0, 0, 0);
            }
            ng_floatx16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[kh][s], bf[kh][s], acc, 0, 0, 0);
            if (interior) {
                if (col_ok) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float xn = old[v] + sign * acc[v];
                        *reinterpret_cast<ng_gfloat*>(ng_uniform_ptr(Xr + (uint32_t)(8 * (v >> 2) + (v & 3)) * ldx4) + offX) = xn;
                        if (fuse == 2) ssq += xn * xn;
                        old[v] = xn;
                    }
                    if (fuse == 2 && col == dim - 1) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) t.wcol[q * n + r0 + 8 * (v >> 2) + (v & 3) + 4 * h] = old[v];
                    }
                }
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rr = r0 + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (rr < rend && col_ok) {
                        const float xn = old[v] + sign * acc[v];
                        X[(int64_t)rr * ldx + col] = xn;
                        if (fuse == 2) {
                            ssq += xn * xn;
                            if (col == dim - 1) t.wcol[q * n + rr] = xn;
                        }
                    }
                }
            }
        }
        if constexpr (WITHY) {
            float* __restrict__ Pp = yt.P[slot] + (int64_t)blockIdx.y * yt.p_chunk + (int64_t)b * yt.y_b[slot];
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = 32 * kh + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (i < rank && col_ok) Pp[(int64_t)i * ldR + col] = yacc[kh][v];
                }
        }
    }
    if (fuse != 0) {      // (uniform over the workgroup: every wavefront reaches the barriers)
        const double tot = block_sum_d((double)ssq, sh);
        double* __restrict__ pr = t.part + q * kNgParts + (int64_t)blockIdx.y * g.maxblk;
        if (threadIdx.x == 0) pr[xb] = tot;
        if (xb == nblk - 1)
            for (int i = nblk + (int)threadIdx.x; i < g.maxblk; i += 256) pr[i] = 0.0;
    }
}

// Y = alpha (sum of the `nchunks` partial products H^T X the first rank update left) + diag(coef1) R for every slot
__global__ __launch_bounds__(256) void ng_y_reduce_slots_kernel(NgSlots t, NgYTable yt, float alpha, int nchunks) {
    const int slot = blockIdx.y, b = blockIdx.z;
    const int dim = t.dim[slot], rank = t.rank;
    const int64_t q = (int64_t)slot * t.batch + b;
    const int ld = (dim + 3) / 4 * 4, ld4 = ld / 4;
    const float* __restrict__ R = reinterpret_cast<const float*>(t.state[slot] + (int64_t)b * t.st_b);
    const float* __restrict__ cf = t.coef + q * (3 * kMaxRank) + kMaxRank;
    const float* __restrict__ P = yt.P[slot] + (int64_t)b * yt.y_b[slot];
    float* __restrict__ Y = yt.Y[slot] + (int64_t)b * yt.y_b[slot];
    for (int e = blockIdx.x * 256 + threadIdx.x; e < rank * ld4; e += gridDim.x * 256) {
        const int i = e / ld4, col = (e - i * ld4) * 4;
        float4 a = *reinterpret_cast<const float4*>(P + (int64_t)e * 4);
        for (int c = 1; c < nchunks; ++c) {
            const float4 v = *reinterpret_cast<const float4*>(P + (int64_t)c * yt.p_chunk + (int64_t)e * 4);
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        const float4 r = *reinterpret_cast<const float4*>(R + (int64_t)e * 4);
        const float ci = cf[i];
        float* y = Y + (int64_t)e * 4;
        if (col + 3 < dim) {
            *reinterpret_cast<float4*>(y) = make_float4(alpha * a.x + ci * r.x, alpha * a.y + ci * r.y, alpha * a.z + ci * r.z, alpha * a.w + ci * r.w);
        } else {        // the padding columns of a row are left alone (their partial products were never written)
            if (col + 0 < dim) y[0] = alpha * a.x + ci * r.x;
            if (col + 1 < dim) y[1] = alpha * a.y + ci * r.y;
            if (col + 2 < dim) y[2] = alpha * a.z + ci * r.z;
        }
    }
}

// Y = alpha H^T X + diag(coef1) R for every slot (the matrix the fold of the state starts from; coef1 = the second
// of the three coefficient vectors).  A workgroup owns 32 columns; its four wavefronts take every fourth tile of 32
// rows: per tile 16 (x KH) v_mfma_f32_32x32x2_f32 with H^T as the A operand (lane i, MFMA step s: H(r0 + 16 h + s, i))
// and X as the B operand (lane j: X(r0 + 16 h + s, c0 + j)), every load a whole 128-byte row segment of H or X per
// half-wavefront through a scalar row pointer and one offset register per matrix.  The four partial products meet in
// LDS and each wavefront finishes 8 of the 32 (x KH) rows.  X is read once, at the pace of the rank updates; the 14
// products of the 440-6x2048-8000 network took two launches of the general GEMM (tiles of 64 rows for 30) and 38 us.
// Columns and rank indices beyond the matrices are clamped for the loads: they reach only accumulator columns
// and rows that are never stored.
template <int KH>
__global__ __launch_bounds__(256) void ng_y_slots_kernel(NgSlots t, NgYTable yt, float alpha) {
    __shared__ float red[4][KH][16 * 64];
    const int slot = blockIdx.y, b = blockIdx.z;
    const int dim = t.dim[slot], n = t.n, rank = t.rank;
    const int c0 = blockIdx.x * 32;
    if (c0 >= dim) return;                              // the grid is as wide as the widest slot (uniform over the workgroup)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, h = lane >> 5, lc = lane & 31;
    const int64_t q = (int64_t)slot * t.batch + b;
    const int col = c0 + lc;
    const bool col_ok = col < dim;
    const int lcc = min(lc, dim - 1 - c0);
    const int64_t ldR = ((int64_t)dim + 3) / 4 * 4, ldx = t.ldx[slot], ldc = t.ldr;
    const uint32_t ldx4 = (uint32_t)ldx * 4u, ldc4 = (uint32_t)ldc * 4u;        // bytes per row
    const float* __restrict__ X = t.x[slot] + (int64_t)b * t.x_b[slot];
    const float* __restrict__ Hm = t.H + q * t.H_b;
    const char* Xc = reinterpret_cast<const char*>(X) + (int64_t)c0 * 4;
    const char* Hc = reinterpret_cast<const char*>(Hm);
    const uint32_t offX = (uint32_t)lcc * 4u + (uint32_t)(16 * h) * ldx4;
    uint32_t offH[KH];
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) offH[kh] = (uint32_t)min(32 * kh + lc, (int)ldc - 1) * 4u + (uint32_t)(16 * h) * ldc4;
    ng_floatx16 acc[KH];
#pragma unroll
    for (int kh = 0; kh < KH; ++kh) acc[kh] = ng_floatx16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r0 = wave * 32; r0 < n; r0 += 128) {
        float bx[16], ah[KH][16];
        if (r0 + 32 <= n) {                             // (uniform)
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                bx[s] = *reinterpret_cast<const ng_gfloat*>(ng_uniform_ptr(Xc + (int64_t)(r0 + s) * ldx4) + offX);
#pragma unroll
                for (int kh = 0; kh < KH; ++kh)
                    ah[kh][s] = *reinterpret_cast<const ng_gfloat*>(ng_uniform_ptr(Hc + (int64_t)(r0 + s) * ldc4) + offH[kh]);
            }
        } else {                                        // the last, ragged tile: per-lane addresses and row checks
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const int r = r0 + 16 * h + s;
                bx[s] = (r < n && col_ok) ? X[(int64_t)r * ldx + col] : 0.f;
#pragma unroll
                for (int kh = 0; kh < KH; ++kh) ah[kh][s] = (r < n && 32 * kh + lc < rank) ? Hm[(int64_t)r * ldc + 32 * kh + lc] : 0.f;
            }
        }
#pragma unroll
        for (int kh = 0; kh < KH; ++kh)
#pragma unroll
            for (int s = 0; s < 16; ++s) acc[kh] = __builtin_amdgcn_mfma_f32_32x32x2f32(ah[kh][s], bx[s], acc[kh], 0, 0, 0);
    }
#pragma unroll
    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][kh][v * 64 + lane] = acc[kh][v];
    __syncthreads();
    // accumulator element v of a lane: rank index 32 kh + 8 (v / 4) + 4 h + v % 4, column c0 + lc; wavefront w finishes v / 4 = w
    const float* __restrict__ R = reinterpret_cast<const float*>(t.state[slot] + (int64_t)b * t.st_b);
    const float* __restrict__ cf = t.coef + q * (3 * kMaxRank) + kMaxRank;
    float* __restrict__ Y = yt.Y[slot] + (int64_t)b * yt.y_b[slot];
#pragma unroll
    for (int kh = 0; kh < KH; ++kh)
#pragma unroll
        for (int vv = 0; vv < 4; ++vv) {
            const int e = (4 * wave + vv) * 64 + lane;
            const float sum = ((red[0][kh][e] + red[1][kh][e]) + red[2][kh][e]) + red[3][kh][e];
            const int i = 32 * kh + 8 * wave + 4 * h + vv;
            if (i < rank && col_ok) Y[(int64_t)i * ldR + col] = alpha * sum + cf[i] * R[(int64_t)i * ldR + col];
        }
}

// Xaug_l[b](r, 0..d) = A_l[b](r, :), Xaug_l[b](r, d) = 1, padding columns 0, for up to kNgSlots / 2 layers
struct NgAugTable {
    const float* A[kNgSlots / 2]; int64_t lda[kNgSlots / 2], a_b[kNgSlots / 2];
    float* X[kNgSlots / 2]; int64_t ldx[kNgSlots / 2], x_b[kNgSlots / 2];
    int d[kNgSlots / 2];
    int n;
};
// With `coef` set the launch has one more row of workgroups (blockIdx.y = the number of layers): workgroup x of that
// row leaves the coefficients of slot x (see ng_coefficients), which depend on the states alone.
__global__ __launch_bounds__(256) void ng_augment_slots_kernel(NgAugTable t, NgSlots sl, float alpha, float eta, int coef) {
    const int l = blockIdx.y, b = blockIdx.z;
    if (coef && l == (int)gridDim.y - 1) {      // (uniform over the workgroup)
        if ((int)blockIdx.x < sl.nslots) ng_coefficients(sl, blockIdx.x, b, alpha, eta);
        return;
    }
    const int64_t ldx = t.ldx[l], lda = t.lda[l];
    const int d = t.d[l];
    const float* __restrict__ A = t.A[l] + (int64_t)b * t.a_b[l];
    float* __restrict__ X = t.X[l] + (int64_t)b * t.x_b[l];
    // a wavefront per row at a time (rows strided over the launch's wavefronts), four columns per lane and trip when
    // both rows are 16-byte aligned: no division per element
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool vec = (lda & 3) == 0 && (ldx & 3) == 0 && (t.a_b[l] & 3) == 0 && (t.x_b[l] & 3) == 0 &&
                     ((reinterpret_cast<uintptr_t>(t.A[l]) | reinterpret_cast<uintptr_t>(t.X[l])) & 15u) == 0;
    for (int r = blockIdx.x * 4 + wave; r < t.n; r += gridDim.x * 4) {
        const float* __restrict__ a = A + (int64_t)r * lda;
        float* __restrict__ x = X + (int64_t)r * ldx;
        if (vec) {
            for (int c0 = 4 * lane; c0 < ldx; c0 += 4 * 256) {       // four trips' loads in flight before their stores
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + 256 * u;
                    if (c + 3 < d) {
                        v[u] = *reinterpret_cast<const float4*>(a + c);
                    } else if (c < ldx) {
                        v[u].x = c + 0 < d ? a[c + 0] : (c + 0 == d ? 1.f : 0.f);
                        v[u].y = c + 1 < d ? a[c + 1] : (c + 1 == d ? 1.f : 0.f);
                        v[u].z = c + 2 < d ? a[c + 2] : (c + 2 == d ? 1.f : 0.f);
                        v[u].w = c + 3 < d ? a[c + 3] : (c + 3 == d ? 1.f : 0.f);
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + 256 * u;
                    if (c < ldx) *reinterpret_cast<float4*>(x + c) = v[u];
                }
            }
        } else {
            for (int c = lane; c < ldx; c += 64) x[c] = c < d ? a[c] : (c == d ? 1.f : 0.f);
        }
    }
}

// ---- host orchestration --------------------------------------------------------------------------

struct NgCall {
    char* state; int64_t st_b;          // bytes between the states of consecutive batch elements
    int dim, rank;
    float* x; int64_t ldx, x_b;         // preconditioned in place
    int n, batch;
    float alpha, eta;
    int mode;                           // 0 apply, 1 apply + fold, 2 three folds first, then apply + fold
    bool scale;                         // multiply by gamma in place (else only report gamma)
    float* gamma;                       // [batch] device floats receiving ||X||/||Xh||
    float* ws;                          // 256-byte aligned scratch of ng_ws(dim, rank, n, batch).total floats
    // Deferred fold (the DNN path finishes the folds of all layers in one batched launch): when defer_Y is set,
    // Y and ||X||^2 of this call are left there and the state is NOT updated by ng_run.
    float* defer_Y = nullptr;           // [batch][RY_b] floats
    double* defer_scal = nullptr;       // [batch][2]
};

#define NG_CHECK(expr)                       \
    do {                                     \
        const int rc__ = (expr);             \
        if (rc__ != 0) return rc__;          \
    } while (0)
#define NG_LAUNCHED() NG_CHECK(note_hip_error(hipGetLastError()))

int ng_eig_smem_bytes(int rank) { return (4 * rank * ((rank + 1) & ~1) + 16) * 8 + 64 * 4; }

// Z = Y Y^T and its eigen-decomposition, new (d, rho, t) and Wt for every (slot, replica) of the table: two launches.
// Reads Y, the squared norms and the old d, rho; does not touch R.
int ng_finish_zeig(const NgFoldTable& tb, int rank, int n, float eta, bool y64, double* Z, double* Wt, int bump, hipStream_t s) {
    // A few workgroups (one per state) on a long chain of dependent LDS accesses and float64 operations, usually
    // launched beside kernels that fill the chip: sharing its compute unit with their workgroups was measured to slow
    // the solver twofold (350 against 180 us for 14 states of rank 30 beside the rank update and the weight-gradient
    // GEMMs; 120 us with the chip to itself), so a launch of few workgroups asks for so much LDS (kEigSoloLds) that no
    // workgroup of a GEMM fits beside it.
    const int need = ng_eig_smem_bytes(rank);
    const int smem = (tb.nslots * tb.batch <= kEigSoloMax && need < kEigSoloLds) ? kEigSoloLds : need;
    if (smem > 64 * 1024) {
        constexpr int kMaxDev = 64;
        static int raised[kMaxDev] = {};    // per device, the largest size allowed so far (benign if two threads race: the call is idempotent)
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) dev = -1;
        if (dev < 0 || raised[dev] < smem) {
            NG_CHECK(note_hip_error(hipFuncSetAttribute(reinterpret_cast<const void*>(ng_eig_kernel),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, smem)));
            if (dev >= 0) raised[dev] = smem;
        }
    }
    const dim3 gz(rank * rank, tb.nslots, tb.batch);
    if (y64) hipLaunchKernelGGL(ng_z_kernel<double>, gz, dim3(256), 0, s, tb, rank, Z);
    else hipLaunchKernelGGL(ng_z_kernel<float>, gz, dim3(256), 0, s, tb, rank, Z);
    NG_LAUNCHED();
    hipLaunchKernelGGL(ng_eig_kernel, dim3(tb.nslots * tb.batch), dim3(kEigThreads), smem, s, tb, rank, n, eta, Z, Wt, bump);
    NG_LAUNCHED();
    return 0;
}

// R <- Wt Y for every (slot, replica) of the table: the one step of a fold that writes R.
int ng_finish_newr(const NgFoldTable& tb, int rank, bool y64, const double* Wt, hipStream_t s) {
    int maxdim = 0;
    for (int i = 0; i < tb.nslots; ++i) if (tb.dim[i] > maxdim) maxdim = tb.dim[i];
    const dim3 gr((unsigned)((maxdim + 3 + 31) / 32), tb.nslots, tb.batch);
    if (y64) hipLaunchKernelGGL(ng_newr_kernel<double>, gr, dim3(256), 0, s, tb, rank, Wt);
    else hipLaunchKernelGGL(ng_newr_kernel<float>, gr, dim3(256), 0, s, tb, rank, Wt);
    NG_LAUNCHED();
    return 0;
}

int ng_finish(const NgFoldTable& tb, int rank, int n, float eta, bool y64, double* Z, double* Wt, int bump, hipStream_t s) {
    NG_CHECK(ng_finish_zeig(tb, rank, n, eta, y64, Z, Wt, bump, s));
    return ng_finish_newr(tb, rank, y64, Wt, s);
}

// Host side of the steps of the apply for a table of slots.
int ng_slots_norms(const NgSlots& t, int which, float alpha, float eta, hipStream_t s) {
    hipLaunchKernelGGL(ng_sumsq_partial_slots_kernel, dim3(256, t.nslots, t.batch), dim3(256), 0, s, t,
                       (which == 1 && t.wcol != nullptr) ? 1 : 0);
    NG_LAUNCHED();
    hipLaunchKernelGGL(ng_sumsq_final_slots_kernel, dim3(t.nslots, t.batch), dim3(256), 0, s, t, which, alpha, eta, 256,
                       which == 0 ? 3 : 1);
    NG_LAUNCHED();
    return 0;
}

// Hout = X R^T for every slot: one launch over the chunks of all contractions (P: [chunk][replica][n x ldr]
// partial products), then their sums
int ng_slots_gemm_H(const NgSlots& t, float* P, float* Hout, hipStream_t s, bool combine = false) {
    GemmDesc g[kThinMaxProblems];
    NgChunkTable ct = {};
    int np = 0, pi = 0;                               // descriptors pending, problems so far
    for (int j = 0; j < t.nslots; ++j) {
        const int dim = t.dim[j], kc = ng_chunk_len(dim), nch = ng_chunk_count(dim);
        ct.first[j] = pi; ct.count[j] = nch;
        for (int c = 0; c < nch; ++c, ++pi) {
            GemmDesc& q = g[np];
            q = GemmDesc();
            q.M = t.n; q.N = t.rank; q.K = (c + 1 < nch) ? kc : dim - c * kc; q.batch = t.batch;
            q.A = t.x[j] + (int64_t)c * kc; q.lda = t.ldx[j]; q.a_bstride = t.x_b[j]; q.a_kc = true;
            q.B = reinterpret_cast<const float*>(t.state[j]) + (int64_t)c * kc; q.ldb = round_up(dim, 4);
            q.b_bstride = t.st_b / 4; q.b_kc = true;
            q.C = P + (int64_t)pi * t.batch * t.H_b; q.ldc = t.ldr; q.c_bstride = t.H_b;
            if (++np == kThinMaxProblems) {
                NG_CHECK(gemm_launch_grouped(g, np, s, true));
                np = 0;
            }
        }
    }
    if (np > 0) NG_CHECK(gemm_launch_grouped(g, np, s, true));
    int64_t gx = ((int64_t)t.n * t.ldr / 4 + 255) / 256;
    if (gx > 64) gx = 64;
    hipLaunchKernelGGL(ng_sum_chunks_slots_kernel, dim3((unsigned)gx, t.nslots, t.batch), dim3(256), 0, s, t, ct, P, Hout, combine ? 1 : 0);
    NG_LAUNCHED();
    return 0;
}

constexpr int kRuRows = 128;          // rows a wavefront of a rank update walks with its block of R in registers
constexpr int kYChunksMax = 8;        // partial products H^T X (one per kRuRows rows) a backward pass keeps at most
inline int ng_ru_row_chunks(int n) { return (n + kRuRows - 1) / kRuRows; }

// X <- X + sign * (H or H2) R for every slot
// fuse: see the kernel; *nparts (when asked for) receives the number of partial sums of squares per (slot, replica)
// the launch leaves.
int ng_slots_rank_update(const NgSlots& t, int use_h2, float sign, hipStream_t s, int fuse = 0, int* nparts = nullptr,
                         const NgYTable* yt = nullptr) {
    NgRuGrid g = {};
    for (int j = 0; j < t.nslots; ++j) {
        const int nb = (t.dim[j] + 127) / 128;
        g.start[j + 1] = g.start[j] + nb;
        if (nb > g.maxblk) g.maxblk = nb;
    }
    const dim3 grid((unsigned)g.start[t.nslots], (unsigned)((t.n + kRuRows - 1) / kRuRows), (unsigned)t.batch);
    if (nparts) *nparts = (int)(g.maxblk * grid.y);
    if (yt != nullptr && (fuse != 1 || use_h2 != 0)) return note_hip_error(hipErrorInvalidValue);
    const NgYTable none = {};
    auto launch = [&](auto khc, auto fusec) {
        constexpr int KH = decltype(khc)::value, FUSE = decltype(fusec)::value;
        hipLaunchKernelGGL((ng_rank_update_slots_kernel<KH, FUSE, false>), grid, dim3(256), 0, s, t, use_h2, sign, kRuRows, none, g);
    };
    auto launch_kh = [&](auto khc) {
        constexpr int KH = decltype(khc)::value;
        if (fuse == 0) launch(khc, std::integral_constant<int, 0>{});
        else if (fuse == 1 && yt != nullptr)
            hipLaunchKernelGGL((ng_rank_update_slots_kernel<KH, 1, true>), grid, dim3(256), 0, s, t, use_h2, sign, kRuRows, *yt, g);
        else if (fuse == 1) launch(khc, std::integral_constant<int, 1>{});
        else launch(khc, std::integral_constant<int, 2>{});
    };
    if (t.rank <= 32) launch_kh(std::integral_constant<int, 1>{});
    else launch_kh(std::integral_constant<int, 2>{});
    NG_LAUNCHED();
    return 0;
}
inline bool ng_parts_fit(const NgSlots& t) {
    int maxdim = 0;
    for (int j = 0; j < t.nslots; ++j) if (t.dim[j] > maxdim) maxdim = t.dim[j];
    return (int64_t)((maxdim + 127) / 128) * ((t.n + kRuRows - 1) / kRuRows) <= kNgParts;
}

int ng_run(const NgCall& c, hipStream_t s) {
    const NgWs w = ng_ws(c.dim, c.rank, c.n, c.batch);
    float* Y = c.defer_Y ? c.defer_Y : c.ws + w.off_Y;
    double* scal = c.defer_scal ? c.defer_scal : reinterpret_cast<double*>(c.ws + w.off_scal);
    double* Z = reinterpret_cast<double*>(c.ws + w.off_Z);
    double* Wt = reinterpret_cast<double*>(c.ws + w.off_Wt);
    double* H64 = reinterpret_cast<double*>(c.ws + w.off_H64);
    double* Y64 = reinterpret_cast<double*>(c.ws + w.off_Y64);
    float* gws = c.ws + w.off_gemm;
    float* P = c.ws + w.off_P;
    const float* Rm = reinterpret_cast<const float*>(c.state);
    const int64_t st_bf = c.st_b / 4;
    NgSlots t;                                       // a table of one slot
    t.state[0] = c.state; t.x[0] = c.x; t.ldx[0] = c.ldx; t.x_b[0] = c.x_b; t.dim[0] = c.dim;
    t.st_b = c.st_b; t.nslots = 1; t.batch = c.batch; t.n = c.n; t.rank = c.rank;
    t.H = c.ws + w.off_H; t.H2 = c.ws + w.off_H2; t.ldr = w.ldr; t.H_b = w.H_b;
    t.coef = c.ws + w.off_coef;
    t.part = reinterpret_cast<double*>(c.ws + w.off_part);
    t.scal = scal;
    t.gamma = c.gamma;
    auto gemm_Y = [&]() -> int {         // Y = (eta/n) H^T X + (1-eta)(diag(d)+rho I) R
        GemmDesc g;
        g.M = c.rank; g.N = c.dim; g.K = c.n; g.batch = c.batch;
        g.A = t.H; g.lda = w.ldr; g.a_bstride = w.H_b; g.a_kc = false;
        g.a_pad4 = true;                 // rows of H are ldr = round_up(rank, 4) floats long
        g.B = c.x; g.ldb = c.ldx; g.b_bstride = c.x_b; g.b_kc = false;
        g.b_pad4 = c.ldx >= w.ld;
        g.C = Y; g.ldc = w.ld; g.c_bstride = w.RY_b;
        g.epi.kind = EPI_ROWSCALE_ADD; g.epi.alpha = c.eta / (float)c.n;
        g.epi.rowvec = t.coef + kMaxRank; g.epi.rowvec_bstride = w.coef_b;
        g.epi.aux = Rm; g.epi.ldaux = w.ld; g.epi.aux_bstride = st_bf;
        return gemm_launch(g, gws, w.gemm_floats, s);
    };
    auto finish_fold = [&](int bump, bool y64) -> int {     // from Y: Z, eigen-decomposition, new state
        NgFoldTable tb;
        tb.state[0] = c.state; tb.st_b = c.st_b; tb.dim[0] = c.dim; tb.scal[0] = scal;
        tb.Y[0] = y64 ? static_cast<const void*>(Y64) : static_cast<const void*>(Y);
        tb.y_b[0] = y64 ? w.Y64_b / 2 : w.RY_b;
        tb.nslots = 1; tb.batch = c.batch; tb.first = 0;
        return ng_finish(tb, c.rank, c.n, c.eta, y64, Z, Wt, bump, s);
    };
    NG_CHECK(ng_slots_norms(t, 0, c.alpha, c.eta, s));              // ||X||^2 and the coefficients of the state
    if (c.mode == 2) {
        for (int f = 0; f < kInitFolds; ++f) {      // in float64: see ng_h64_kernel
            hipLaunchKernelGGL(ng_h64_kernel, dim3(c.n, c.batch), dim3(256), 0, s, c.state, c.st_b, c.dim, c.rank, c.x, c.ldx, c.x_b,
                               H64, w.H64_b);
            NG_LAUNCHED();
            hipLaunchKernelGGL(ng_y64_kernel, dim3((unsigned)((c.dim + 255) / 256), c.batch), dim3(256), 0, s, c.state, c.st_b, c.dim,
                               c.rank, c.n, c.eta, c.x, c.ldx, c.x_b, H64, w.H64_b, Y64, w.Y64_b);
            NG_LAUNCHED();
            NG_CHECK(finish_fold(0, true));
        }
        // the coefficients again, from the folded state (the partial sums of ||X||^2 are still in place)
        hipLaunchKernelGGL(ng_sumsq_final_slots_kernel, dim3(1, c.batch), dim3(256), 0, s, t, 0, c.alpha, c.eta, 256, 2);
        NG_LAUNCHED();
    }
    NG_CHECK(ng_slots_gemm_H(t, P, t.H, s));
    if (c.mode >= 1) NG_CHECK(gemm_Y());
    NG_CHECK(ng_slots_rank_update(t, 0, -1.f, s));      // X1 = X - H R
    NG_CHECK(ng_slots_gemm_H(t, P, t.H2, s, true));     // H (I - E) - H2, H2 = X1 R^T  (what the first pass left inside the subspace)
    NG_CHECK(ng_slots_rank_update(t, 1, 1.f, s));       // Xh = X1 + (H (I - E) - H2) R
    NG_CHECK(ng_slots_norms(t, 1, c.alpha, c.eta, s));  // ||Xh||^2, gamma
    if (c.scale) {
        int64_t gx = ((int64_t)c.n * c.dim + 255) / 256;
        if (gx > 2048) gx = 2048;
        hipLaunchKernelGGL(ng_scale_kernel, dim3((unsigned)gx, c.batch), dim3(256), 0, s, c.x, c.ldx, c.x_b, c.n, c.dim, c.gamma);
        NG_LAUNCHED();
    }
    if (c.mode >= 1 && !c.defer_Y) NG_CHECK(finish_fold(1, false));
    return 0;
}

}  // namespace

namespace {
// scratch of one layer's update: [augmented input copy | gamma_in | gamma_out | preconditioner scratch]
int64_t ng_layer_ws_floats(int d_in, int d_out, int n, int k, int rank) {
    const int64_t ld_in = round_up(d_in + 1, 4);
    const int64_t a = ng_ws(d_in + 1, rank, n, k).total, b = ng_ws(d_out, rank, n, k).total;
    return round_up((int64_t)k * n * ld_in, 64) + 2 * round_up(k, 64) + (a > b ? a : b);
}
}  // namespace

namespace {
// NG scratch of a whole backward pass (offsets in floats): what survives until the batched fold at the end
// -- Y and the two squared norms of every (layer side, replica), then Z and Wt -- followed by the scratch
// that one layer's update reuses.
struct NgDnnLayout {
    int64_t y_off[2 * 64], y_b[2 * 64];     // slot 2(l-1): input side of layer l, slot 2(l-1)+1: output side
    int64_t y_total, py_off; int py_chunks;  // partial products H^T X per block of rows of the first rank update: py_chunks copies of the Y region (0: not kept)
    int64_t scal_off, z_off, wt_off, layer_off, layer_floats, total;
    // all layers at once: augmented inputs of every layer, then per-(slot, replica) H, H2, coefficients, partial
    // sums and gamma
    int64_t xaug_off[64 + 1], ld_in[64 + 1];
    int64_t ldr, H_b, h_off, h2_off, coef_off, part_off, gamma_off, hp_off, wcol_off;
};
NgDnnLayout ng_dnn_layout(const int* d, int L, int n, int k, int rank) {
    NgDnnLayout y;
    int64_t off = 0;
    for (int l = 1; l <= L; ++l)
        for (int side = 0; side < 2; ++side) {
            const int dim = side == 0 ? d[l - 1] + 1 : d[l];
            const int j = 2 * (l - 1) + side;
            y.y_b[j] = round_up((int64_t)rank * round_up(dim, 4), 64);
            y.y_off[j] = off;
            off += y.y_b[j] * k;
        }
    y.scal_off = off; off += round_up(2 * 2 * (int64_t)(2 * L) * k, 64);
    y.z_off = off;    off += 2 * (int64_t)kMaxRank * kMaxRank * (2 * L) * k;
    y.wt_off = off;   off += 2 * (int64_t)kMaxRank * kMaxRank * (2 * L) * k;
    y.layer_off = off;
    y.layer_floats = 0;
    for (int l = 1; l <= L; ++l) {
        const int64_t f = ng_layer_ws_floats(d[l - 1], d[l], n, k, rank);
        if (f > y.layer_floats) y.layer_floats = f;
    }
    off += y.layer_floats;
    for (int l = 1; l <= L; ++l) {
        y.ld_in[l] = round_up(d[l - 1] + 1, 32);
        y.xaug_off[l] = off;
        off += round_up((int64_t)k * n * y.ld_in[l], 64);
    }
    const int64_t q = (int64_t)2 * L * k;
    y.ldr = round_up(rank, 4);
    y.H_b = round_up((int64_t)n * y.ldr, 64);
    y.h_off = off;     off += q * y.H_b;
    y.h2_off = off;    off += q * y.H_b;
    y.coef_off = off;  off += q * 3 * kMaxRank;
    y.part_off = off;  off += q * 2 * kNgParts;
    y.gamma_off = off; off += round_up(q, 64);
    int64_t nprob = 0;
    for (int l = 1; l <= L; ++l) nprob += ng_chunk_count(d[l - 1] + 1) + ng_chunk_count(d[l]);
    y.hp_off = off;    off += nprob * k * y.H_b;
    y.wcol_off = off;  off += round_up(q * n, 64);
    y.y_total = y.scal_off;                            // the Y region starts the layout
    y.py_chunks = ng_ru_row_chunks(n) <= kYChunksMax ? ng_ru_row_chunks(n) : 0;
    y.py_off = off;    off += (int64_t)y.py_chunks * y.y_total;
    y.total = off;
    return y;
}
}  // namespace

int64_t ng_dnn_ws_floats(const int* d, int L, int n, int k, int rank) { return ng_dnn_layout(d, L, n, k, rank).total; }

namespace {
// The fold table of slots [j0, j0 + nslots) of a network's 2 L layer sides.
NgFoldTable ng_dnn_fold_table(const NgDnnLayout& y, const int* d, int L, int k, char* ng_state, int64_t state_stride, float* ws, int j0) {
    double* scal = reinterpret_cast<double*>(ws + y.scal_off);
    NgFoldTable tb;
    tb.nslots = (2 * L - j0) < kNgSlots ? (2 * L - j0) : kNgSlots;
    tb.batch = k; tb.first = j0; tb.st_b = (int64_t)2 * L * state_stride;
    for (int i = 0; i < tb.nslots; ++i) {
        const int j = j0 + i, l = j / 2 + 1;
        tb.state[i] = ng_state + (int64_t)j * state_stride;
        tb.dim[i] = (j % 2 == 0) ? d[l - 1] + 1 : d[l];
        tb.Y[i] = ws + y.y_off[j];
        tb.y_b[i] = y.y_b[j];
        tb.scal[i] = scal + (int64_t)j * k * 2;
    }
    return tb;
}

// One internal stream and three events per host thread and device, created on first use and kept until the
// process ends (default priority, no timing): the folds of the Fisher states run there beside the weight update.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    bool ok = false, tried = false;
};
SideStream* side_stream() {
    constexpr int kMaxDev = 64;
    static thread_local SideStream table[kMaxDev];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return nullptr;
    SideStream& ss = table[dev];
    if (!ss.tried) {
        ss.tried = true;
        const char* serial = getenv("MAVG_NG_SERIAL_FOLD");       // "1": keep every launch on the caller's stream
        if (serial && serial[0] == '1') return nullptr;
        bool good = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess;
        for (int i = 0; i < 3 && good; ++i) good = hipEventCreateWithFlags(&ss.ev[i], hipEventDisableTiming) == hipSuccess;
        if (!good) (void)hipGetLastError();      // fall back to the caller's stream alone
        ss.ok = good;
    }
    return ss.ok ? &ss : nullptr;
}
}  // namespace

// Finish the folds of all layer sides and replicas of one backward pass (three launches per 32 slots).
int ng_dnn_finish(const int* d, int L, int n, int k, int rank, float eta, char* ng_state, int64_t state_stride, float* ws,
                  hipStream_t s) {
    const NgDnnLayout y = ng_dnn_layout(d, L, n, k, rank);
    double* Z = reinterpret_cast<double*>(ws + y.z_off);
    double* Wt = reinterpret_cast<double*>(ws + y.wt_off);
    for (int j0 = 0; j0 < 2 * L; j0 += kNgSlots) {
        const NgFoldTable tb = ng_dnn_fold_table(y, d, L, k, ng_state, state_stride, ws, j0);
        NG_CHECK(ng_finish(tb, rank, n, eta, false, Z, Wt, 1, s));
    }
    return 0;
}

int ng_layer_update(const NgLayerArgs& a, hipStream_t s) {
    const NgDnnLayout lay = ng_dnn_layout(a.dims, a.L, a.n, a.k, a.rank);
    if (a.ws_floats < lay.total) return (int)hipErrorInvalidValue;
    const int dim_in = a.d_in + 1;
    const int64_t ld_in = round_up(dim_in, 4);
    const int64_t aug_b = (int64_t)a.n * ld_in;
    const int j_in = 2 * (a.l - 1), j_out = j_in + 1;
    double* scal = reinterpret_cast<double*>(a.ws + lay.scal_off);
    float* Xaug = a.ws + lay.layer_off;
    float* gamma_in = Xaug + round_up((int64_t)a.k * aug_b, 64);
    float* gamma_out = gamma_in + round_up(a.k, 64);
    float* ngws = gamma_out + round_up(a.k, 64);
    {
        int64_t gx = (a.n + 3) / 4;       // a wavefront per row
        if (gx > 2048) gx = 2048;
        NgAugTable au;
        au.A[0] = a.A_in; au.lda[0] = a.a_ld; au.a_b[0] = a.a_bstride; au.d[0] = a.d_in;
        au.X[0] = Xaug; au.ldx[0] = ld_in; au.x_b[0] = aug_b; au.n = a.n;
        hipLaunchKernelGGL(ng_augment_slots_kernel, dim3((unsigned)gx, 1, a.k), dim3(256), 0, s, au, NgSlots(), 0.f, 0.f, 0);
        NG_LAUNCHED();
    }
    NgCall c;
    c.rank = a.rank; c.n = a.n; c.batch = a.k; c.alpha = a.alpha; c.eta = a.eta; c.mode = a.mode; c.scale = false;
    c.ws = ngws;
    c.state = a.state_in; c.st_b = a.state_rstride; c.dim = dim_in; c.x = Xaug; c.ldx = ld_in; c.x_b = aug_b; c.gamma = gamma_in;
    c.defer_Y = a.ws + lay.y_off[j_in]; c.defer_scal = scal + (int64_t)j_in * a.k * 2;
    NG_CHECK(ng_run(c, s));
    c.state = a.state_out; c.dim = a.d_out; c.x = a.delta; c.ldx = a.ldd; c.x_b = a.d_bstride; c.gamma = gamma_out;
    c.defer_Y = a.ws + lay.y_off[j_out]; c.defer_scal = scal + (int64_t)j_out * a.k * 2;
    NG_CHECK(ng_run(c, s));
    {   // [W | b] <- [W | b] - lr g_out g_in  Xh_out^T Xh_in : the last column of the product is the bias update
        GemmDesc g;
        g.M = a.d_out; g.N = a.d_in + 1; g.K = a.n; g.batch = a.k;
        g.A = a.delta; g.lda = a.ldd; g.a_bstride = a.d_bstride; g.a_kc = false;
        g.a_pad4 = true;       // rows of delta are round_up(d_out, 4) floats long
        g.B = Xaug; g.ldb = ld_in; g.b_bstride = aug_b; g.b_kc = false;
        g.b_pad4 = true;       // rows of Xaug are ld_in = round_up(d_in + 1, 4) floats long
        g.C = a.W; g.ldc = a.d_in; g.c_bstride = a.theta_stride;
        g.epi.kind = EPI_AXPBY; g.epi.alpha = -a.lr; g.epi.beta = 1.f;
        g.epi.alpha_dev0 = gamma_in; g.epi.alpha_dev1 = gamma_out;
        g.epi.lastcol = a.d_in; g.epi.lastcol_dst = a.b; g.epi.lastcol_bstride = a.theta_stride;
        NG_CHECK(gemm_launch(g, a.gemm_ws, a.gemm_ws_floats, s));
    }
    return 0;
}


// The preconditioned update of every layer (steady state: one fold per minibatch), a fixed number of launches
// whatever the depth: augment, ||X||^2 + coefficients, H, Y, X1, H2 (combined with H where its chunks are summed), Xh, ||Xh||^2 + gamma, then the weight
// gradients of all layers as one grouped launch.  The folds stay pending until ng_dnn_finish.
int ng_dnn_update(const NgLayerArgs* layers, int L, char* ng_state, int64_t state_stride, hipStream_t s) {
    const NgLayerArgs& a0 = layers[0];
    const int n = a0.n, k = a0.k, rank = a0.rank;
    const NgDnnLayout lay = ng_dnn_layout(a0.dims, L, n, k, rank);
    if (a0.ws_floats < lay.total) return (int)hipErrorInvalidValue;
    float* ws = a0.ws;
    // The fold (Z = Y Y^T, its eigen-decomposition, R <- Wt Y) needs only Y, the squared norms and the old state, and
    // is a chain of small, latency-bound launches (14 workgroups in the eigen-solver): with all layers in one pass it
    // runs on the internal stream beside the rest of the apply and the weight update, which occupy the whole chip.
    // Its last step, the only one that writes R, waits until the apply has read R for the last time; the caller's
    // stream waits for it before this call's work is complete.  (Forking only once, behind the second rank update,
    // would spare the caller's stream one record of an event, about 6 us between two launches, but was measured
    // slower by 90 us: a launch of the internal stream that arrives while the weight-gradient launch holds every
    // compute unit gets its workgroups placed only as that launch drains.)
    SideStream* side = (a0.mode == 1 && L <= kNgSlots / 2) ? side_stream() : nullptr;
    double* Zf = reinterpret_cast<double*>(ws + lay.z_off);
    double* Wtf = reinterpret_cast<double*>(ws + lay.wt_off);
    double* scal = reinterpret_cast<double*>(ws + lay.scal_off);
    constexpr int kLayersPerPass = kNgSlots / 2;
    for (int l0 = 0; l0 < L; l0 += kLayersPerPass) {
        const int nl = (L - l0) < kLayersPerPass ? (L - l0) : kLayersPerPass;
        const int j0 = 2 * l0;                          // first slot of this pass
        NgSlots t;
        NgAugTable au;
        t.nslots = 2 * nl; t.batch = k; t.n = n; t.rank = rank; t.st_b = a0.state_rstride;
        t.ldr = lay.ldr; t.H_b = lay.H_b;
        t.H = ws + lay.h_off + (int64_t)j0 * k * lay.H_b;
        t.H2 = ws + lay.h2_off + (int64_t)j0 * k * lay.H_b;
        t.coef = ws + lay.coef_off + (int64_t)j0 * k * 3 * kMaxRank;
        t.part = reinterpret_cast<double*>(ws + lay.part_off) + (int64_t)j0 * k * kNgParts;
        t.scal = scal + (int64_t)j0 * k * 2;
        t.gamma = ws + lay.gamma_off + (int64_t)j0 * k;
        t.wcol = ws + lay.wcol_off + (int64_t)j0 * k * n;
        au.n = n;
        for (int i = 0; i < nl; ++i) {
            const NgLayerArgs& a = layers[l0 + i];
            const int l = a.l;
            const int64_t ld_in = lay.ld_in[l], aug_b = (int64_t)n * ld_in;
            float* Xaug = ws + lay.xaug_off[l];
            au.A[i] = a.A_in; au.lda[i] = a.a_ld; au.a_b[i] = a.a_bstride; au.d[i] = a.d_in;
            au.X[i] = Xaug; au.ldx[i] = ld_in; au.x_b[i] = aug_b;
            t.state[2 * i] = a.state_in;      t.x[2 * i] = Xaug;        t.ldx[2 * i] = ld_in;     t.x_b[2 * i] = aug_b;
            t.dim[2 * i] = a.d_in + 1;
            t.state[2 * i + 1] = a.state_out; t.x[2 * i + 1] = a.delta; t.ldx[2 * i + 1] = a.ldd; t.x_b[2 * i + 1] = a.d_bstride;
            t.dim[2 * i + 1] = a.d_out;
        }
        // The two rank updates take the norms with them (||X||^2 as the first one reads X, ||Xh||^2 as the second one
        // writes it) whenever the per-workgroup partial sums fit their table: two passes over the matrices fewer.  Then
        // the coefficients, which depend on the states alone, are left by one more row of workgroups of the launch
        // that augments the inputs.
        const bool fused = ng_parts_fit(t);
        {
            int64_t gx = (n + 3) / 4;         // a wavefront per row
            if (gx > 1024) gx = 1024;
            if (gx < t.nslots) gx = t.nslots;
            hipLaunchKernelGGL(ng_augment_slots_kernel, dim3((unsigned)gx, nl + (fused ? 1 : 0), k), dim3(256), 0, s, au, t,
                               a0.alpha, a0.eta, fused ? 1 : 0);
            NG_LAUNCHED();
        }
        float* P = ws + lay.hp_off;                      // partial products [problem][replica][n x ldr]
        int nparts = 0;
        if (!fused) NG_CHECK(ng_slots_norms(t, 0, a0.alpha, a0.eta, s));
        NG_CHECK(ng_slots_gemm_H(t, P, t.H, s));
        // Y = (eta/n) H^T X + (1-eta)(diag(d)+rho I) R for every slot, left where ng_dnn_finish expects it: the product
        // is taken by the first rank update as it reads X (one partial product per block of kRuRows rows, summed by a
        // small launch), or by a pass of its own where those partial products have no room.
        NgYTable yt = {};
        int maxdim = 0;
        for (int j = 0; j < t.nslots; ++j) {
            yt.Y[j] = ws + lay.y_off[j0 + j]; yt.y_b[j] = lay.y_b[j0 + j];
            yt.P[j] = ws + lay.py_off + lay.y_off[j0 + j];
            if (t.dim[j] > maxdim) maxdim = t.dim[j];
        }
        yt.p_chunk = lay.y_total;
        const bool with_y = a0.mode >= 1, fuse_y = with_y && fused && lay.py_chunks > 0;
        if (with_y && !fuse_y) {
            const dim3 gy((unsigned)((maxdim + 31) / 32), (unsigned)t.nslots, (unsigned)k);
            if (rank <= 32) hipLaunchKernelGGL(ng_y_slots_kernel<1>, gy, dim3(256), 0, s, t, yt, a0.eta / (float)n);
            else hipLaunchKernelGGL(ng_y_slots_kernel<2>, gy, dim3(256), 0, s, t, yt, a0.eta / (float)n);
            NG_LAUNCHED();
        }
        // (Moving the two small launches that only the fold needs at this point - the sum of the partial products and
        // the sum of the shares of ||X||^2 - to the internal stream as well was measured and made no difference.)
        if (fused) {                                         // X1 = X - H R, and ||X||^2 (and H^T X)
            NG_CHECK(ng_slots_rank_update(t, 0, -1.f, s, 1, &nparts, fuse_y ? &yt : nullptr));
            if (fuse_y) {
                int gx = (rank * ((maxdim + 3) / 4) + 255) / 256;
                if (gx > 256) gx = 256;
                hipLaunchKernelGGL(ng_y_reduce_slots_kernel, dim3((unsigned)gx, (unsigned)t.nslots, (unsigned)k), dim3(256), 0, s, t, yt,
                                   a0.eta / (float)n, lay.py_chunks);
                NG_LAUNCHED();
            }
            hipLaunchKernelGGL(ng_sumsq_final_slots_kernel, dim3(t.nslots, t.batch), dim3(256), 0, s, t, 0, a0.alpha, a0.eta, nparts, 1);
            NG_LAUNCHED();
        } else {
            NG_CHECK(ng_slots_rank_update(t, 0, -1.f, s));
        }
        if (a0.mode >= 1 && side) {      // Y and ||X||^2 are there: the fold may start
            NG_CHECK(note_hip_error(hipEventRecord(side->ev[0], s)));
            NG_CHECK(note_hip_error(hipStreamWaitEvent(side->stream, side->ev[0], 0)));
            const NgFoldTable tb = ng_dnn_fold_table(lay, a0.dims, L, k, ng_state, state_stride, ws, 0);
            NG_CHECK(ng_finish_zeig(tb, rank, n, a0.eta, false, Zf, Wtf, 1, side->stream));
        }
        NG_CHECK(ng_slots_gemm_H(t, P, t.H2, s, true));      // H (I - E) - H2, H2 = X1 R^T: combined where the chunks are summed
        NG_CHECK(ng_slots_rank_update(t, 1, 1.f, s, fused ? 2 : 0, &nparts));     // Xh = X1 + (H (I - E) - H2) R (, ||Xh||^2, last column)
        if (side) {      // R has been read for the last time: the fold may write it
            NG_CHECK(note_hip_error(hipEventRecord(side->ev[1], s)));
            NG_CHECK(note_hip_error(hipStreamWaitEvent(side->stream, side->ev[1], 0)));
            const NgFoldTable tb = ng_dnn_fold_table(lay, a0.dims, L, k, ng_state, state_stride, ws, 0);
            NG_CHECK(ng_finish_newr(tb, rank, false, Wtf, side->stream));
            NG_CHECK(note_hip_error(hipEventRecord(side->ev[2], side->stream)));
        }
        if (fused) {
            hipLaunchKernelGGL(ng_sumsq_final_slots_kernel, dim3(t.nslots, t.batch), dim3(256), 0, s, t, 1, a0.alpha, a0.eta, nparts, 1);
            NG_LAUNCHED();
        } else {
            NG_CHECK(ng_slots_norms(t, 1, a0.alpha, a0.eta, s));
        }
        {   // W <- W - lr g_out g_in Xh_out^T Xh_in[:, :d_in] for the layers of this pass, and as the weighted row sums
            // of the same launch b <- b - lr g_out g_in Xh_out^T Xh_in[:, d_in] (the preconditioned "ones" column,
            // left contiguous by the pass that took the norms)
            GemmDesc g[kLayersPerPass];
            for (int i = 0; i < nl; ++i) {
                const NgLayerArgs& a = layers[l0 + i];
                GemmDesc& q = g[i];
                q.M = a.d_out; q.N = a.d_in; q.K = n; q.batch = k;
                q.A = a.delta; q.lda = a.ldd; q.a_bstride = a.d_bstride; q.a_kc = false;
                q.a_pad4 = true;
                q.B = t.x[2 * i]; q.ldb = t.ldx[2 * i]; q.b_bstride = t.x_b[2 * i]; q.b_kc = false;
                q.b_pad4 = true;
                q.C = a.W; q.ldc = a.d_in; q.c_bstride = a.theta_stride;
                q.epi.kind = EPI_AXPBY; q.epi.alpha = -a.lr; q.epi.beta = 1.f;
                q.epi.alpha_dev0 = t.gamma + (int64_t)(2 * i) * k; q.epi.alpha_dev1 = t.gamma + (int64_t)(2 * i + 1) * k;
                q.epi.rowsum_dst = a.b; q.epi.rowsum_bstride = a.theta_stride; q.epi.rowsum_alpha = -a.lr; q.epi.rowsum_beta = 1.f;
                q.epi.rowsum_w = t.wcol + (int64_t)(2 * i) * k * n; q.epi.rowsum_w_bstride = n;
            }
            NG_CHECK(gemm_launch_grouped(g, nl, s));
        }
    }
    if (side) NG_CHECK(note_hip_error(hipStreamWaitEvent(s, side->ev[2], 0)));
    else if (a0.mode == 1) NG_CHECK(ng_dnn_finish(a0.dims, L, n, k, rank, a0.eta, ng_state, state_stride, ws, s));
    return 0;
}

}  // namespace mavg

using namespace mavg;

extern "C" int64_t ngsgd_state_bytes(int32_t dim, int32_t rank) {
    if (dim < 2 || rank < 1 || rank > kMaxRank || rank >= dim) return MAVG_E_DIM;
    const int64_t ld = ((int64_t)dim + 3) / 4 * 4;
    return round_up((int64_t)rank * ld * 4 + (int64_t)rank * 8 + 24, 16);
}

extern "C" int64_t ngsgd_workspace_bytes(int32_t dim, int32_t rank, int32_t n) {
    if (dim < 2 || rank < 1 || rank > kMaxRank || rank >= dim || n < 1) return MAVG_E_DIM;
    return ng_ws(dim, rank, n, 1).total * 4 + 256;
}

extern "C" int32_t ngsgd_state_init(void* state, int32_t dim, int32_t rank, void* stream) {
    if (!state) return MAVG_E_NULL;
    if (dim < 2 || rank < 1 || rank > kMaxRank || rank >= dim) return MAVG_E_DIM;
    if (reinterpret_cast<uintptr_t>(state) & 15u) return MAVG_E_ALIGN;
    const int64_t work = (int64_t)rank * (((int64_t)dim + 3) / 4 * 4);
    int64_t gx = (work + 255) / 256;
    if (gx > 1024) gx = 1024;
    hipLaunchKernelGGL(ng_init_kernel, dim3((unsigned)gx), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<char*>(state), dim, rank);
    return note_hip_error(hipGetLastError()) == 0 ? MAVG_OK : MAVG_E_LAUNCH;
}

extern "C" int32_t ngsgd_precondition(void* state, int32_t dim, int32_t rank, float* x, int64_t ldx, int32_t n, float alpha,
                                      float eta, int32_t update, void* workspace, int64_t workspace_bytes, void* stream) {
    if (!state || !x) return MAVG_E_NULL;
    if (dim < 2 || rank < 1 || rank > kMaxRank || rank >= dim || n < 1) return MAVG_E_DIM;
    if (update < 0 || update > 2) return MAVG_E_FLAG;
    if (!(alpha > 0.f) || !(eta > 0.f && eta < 1.f)) return MAVG_E_DIM;
    if ((reinterpret_cast<uintptr_t>(state) & 15u) || (reinterpret_cast<uintptr_t>(x) & 15u) || ldx < dim) return MAVG_E_ALIGN;
    const NgWs w = ng_ws(dim, rank, n, 1);
    if (!workspace || workspace_bytes < w.total * 4 + 256) return MAVG_E_WORKSPACE;
    NgCall c;
    c.state = static_cast<char*>(state); c.st_b = 0; c.dim = dim; c.rank = rank;
    c.x = x; c.ldx = ldx; c.x_b = 0; c.n = n; c.batch = 1; c.alpha = alpha; c.eta = eta; c.mode = update; c.scale = true;
    c.ws = reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~uintptr_t(255));
    c.gamma = c.ws + w.off_gamma;
    return ng_run(c, static_cast<hipStream_t>(stream)) == 0 ? MAVG_OK : MAVG_E_LAUNCH;
}
