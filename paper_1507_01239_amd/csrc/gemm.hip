// fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32) with the fused epilogues the training path
// needs and a deterministic split of the contraction for problems with too few output tiles to fill 256
// compute units.
//
// This file: the plan (tile shape, splits), the dispatch to the kernel families, the split-contraction reducer and
// the exported entry points.  The kernels live in gemm_device.h and are instantiated per family in
// gemm_dma64.hip, gemm_dma128.hip, gemm_kg.hip and gemm_legacy.hip (separate files so that they compile in parallel).
//
// Two families of kernels share the epilogues, the tile order and the split-contraction reducer:
//  - gemm_dma_kernel: 64x64 tiles whose operands go from global memory straight into an LDS ring
//    (global_load_lds_dwordx4); the kernel of the training step whenever the loads need no masking;
//  - gemm_kernel<BM,BN,BK,...>: register-staged tiles of several shapes, with guarded loads for ragged and
//    unaligned operands.  One workgroup = WM x WN wavefronts over a BM x BN tile, each wavefront owning a grid
//    of 32x32 MFMA accumulators; operand tiles staged in LDS k-major ([k][m], [k][n]), double-buffered.
#include "gemm_device.h"
#include "gemm_launchers.h"

namespace mavg {

// Sum the partial results of a split contraction in split order and apply the epilogue.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(GemmKParams p) {
    const int b = blockIdx.y;
    const int64_t MN = (int64_t)p.M * p.N;
    const EpiCtx c = epi_ctx(p.epi, p.C, p.c_bstride, b);
    const float* __restrict__ W = p.ws + (int64_t)b * p.splits * MN;
    if ((p.N & 3) == 0) {
        const int64_t nq = MN >> 2;
        for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += (int64_t)gridDim.x * 256) {
            // request all (at most 16) partial sums before adding any: one memory latency, not one per few splits
            float4 t[16];
#pragma unroll
            for (int sp = 0; sp < 16; ++sp)
                if (sp < p.splits) t[sp] = *reinterpret_cast<const float4*>(W + sp * MN + q * 4);
            float4 s = t[0];
#pragma unroll
            for (int sp = 1; sp < 16; ++sp)
                if (sp < p.splits) { s.x += t[sp].x; s.y += t[sp].y; s.z += t[sp].z; s.w += t[sp].w; }
            for (int sp = 16; sp < p.splits; ++sp) {
                const float4 u = *reinterpret_cast<const float4*>(W + sp * MN + q * 4);
                s.x += u.x; s.y += u.y; s.z += u.z; s.w += u.w;
            }
            const int64_t e = q * 4;
            const int m = (int)(e / p.N), n = (int)(e - (int64_t)m * p.N);
            MAVG_EPI_DISPATCH(p.epi.kind, (epi_apply4<KIND>(p.epi, c, p.ldc, p.N, m, n, s)))
        }
    } else {
        for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < MN; e += (int64_t)gridDim.x * 256) {
            float t[16];
#pragma unroll
            for (int sp = 0; sp < 16; ++sp)
                if (sp < p.splits) t[sp] = W[sp * MN + e];
            float s = t[0];
#pragma unroll
            for (int sp = 1; sp < 16; ++sp)
                if (sp < p.splits) s += t[sp];
            for (int sp = 16; sp < p.splits; ++sp) s += W[sp * MN + e];
            const int m = (int)(e / p.N), n = (int)(e - (int64_t)m * p.N);
            MAVG_EPI_DISPATCH(p.epi.kind, (epi_apply<KIND>(p.epi, c, p.ldc, p.N, m, n, s)))
        }
    }
}

// ---- host side -----------------------------------------------------------------------------------

struct TileCfg { int bm, bn, bk, threads; };
// indexed by GemmCfg
static const TileCfg kCfgs[CFG_COUNT] = {
    {64, 64, 16, 256},     // CFG_64
    {64, 64, 16, 256},     // CFG_64_REG
    {128, 128, 16, 512},   // CFG_128_REG
    {128, 64, 16, 256},    // CFG_128x64
    {64, 128, 16, 256},    // CFG_64x128
    {128, 128, 16, 256},   // CFG_128
    {64, 64, 16, 256},     // CFG_64_RING3
    {32, 64, 16, 512},     // CFG_KG_32x64
    {32, 32, 16, 256},     // CFG_KG_32x32
};
constexpr int kNumCfgs = CFG_COUNT;
static inline bool cfg_dma_only(int cfg) { return cfg >= CFG_128x64 && cfg != CFG_64_RING3; }
static inline bool cfg_kg(int cfg) { return cfg == CFG_KG_32x64 || cfg == CFG_KG_32x32; }

GemmPlan gemm_plan(int M, int N, int K, int batch, int force_cfg, int force_splits) {
    GemmPlan pl;
    // Measured on MI355X (layer shapes at minibatch 256 to 1024, 1 and 8 replicas): the 64x64 direct-to-LDS
    // kernel wins everywhere; many small workgroups per compute unit run out of phase and hide each other's
    // load, barrier and epilogue latencies.
    int cfg = force_cfg;
    // Only GEMMs that are large in all three dimensions (none of the training shapes: there one of the three is
    // the minibatch) gain from 128x128 tiles: 141 against 127 TFLOP/s at 4096^3.
    // A short contraction over many tiles (the weight gradients: K is the minibatch) runs better with a ring of
    // three stages: a quarter less LDS lets one more workgroup share the compute unit, and it is the overlap of
    // one workgroup's read-modify-write epilogue with its neighbours' multiplies that is short there
    // (8000x2048x256: 90 against 95 us); the long contractions want the deeper ring (256x8000x2048: 73 against 81).
    if (cfg < 0 || cfg >= kNumCfgs) {
        const int64_t t64 = (int64_t)((M + 63) / 64) * ((N + 63) / 64) * batch;
        cfg = (M >= 2048 && N >= 2048 && K >= 2048) ? CFG_128 : (K <= 1024 && t64 >= 1024) ? CFG_64_RING3 : CFG_64;
        // A skinny problem whose 32x64 tiles come to about one per compute unit (the 256 x 2048 x 2048 hidden
        // layers of the minibatch-256 step) does its contraction split inside the workgroup: 24.5 against
        // 26.9 us including the reducer (13.1 against 15.9 us for the 440-wide first layer).  Not at half or
        // twice that many tiles, nor for K = 8000 (measured).
        const int64_t t3264 = (int64_t)((M + 31) / 32) * ((N + 63) / 64) * batch;
        // (One workgroup of it fills a compute unit's LDS: past one tile per compute unit the launch takes two turns,
        // 39 us at 272 or 288 rows against 29 us for 64x64 tiles split in three.)
        if (cfg == CFG_64 && t3264 >= 3 * kNumCU / 4 && t3264 <= kNumCU && K >= 256 && K <= 4096) cfg = CFG_KG_32x64;
        // Half as many rows again (128 x 2048 x 2048): 32x32 tiles, one wavefront per k-group, no barrier in the
        // loop: 18.0 against 19.8 us.  (Two of its workgroups share a compute unit.)
        const int64_t t3232 = (int64_t)((M + 31) / 32) * ((N + 31) / 32) * batch;
        if (cfg == CFG_64 && t3232 >= 3 * kNumCU / 4 && t3232 <= kNumCU + kNumCU / 8 && K >= 1024 && K <= 4096) cfg = CFG_KG_32x32;
    }
    pl.cfg = cfg;
    pl.bm = kCfgs[cfg].bm; pl.bn = kCfgs[cfg].bn;
    const int bk = kCfgs[cfg].bk;
    const int64_t tiles = (int64_t)((M + pl.bm - 1) / pl.bm) * ((N + pl.bn - 1) / pl.bn) * batch;
    int splits = cfg_kg(cfg) ? 1 : force_splits;      // these split the contraction inside the workgroup only
    if (splits <= 0) {
        // A launch takes about as long as the workgroups of its fullest compute unit one after the other: in units of
        // contraction steps, ceil(tiles * splits / compute units) * K / splits; a compute unit with a single, short
        // workgroup (fewer than 6000 steps) has nothing to hide its prologue and epilogue behind (+ 20 %); the reducer
        // costs 6 us (340 steps' worth at 64x64) and each split 8 bytes per element of C at about 4 TB/s.  Splits keep at
        // least 16 k-tiles each, and a split must promise 5 % to be taken.  Measured with 64x64 tiles (us for the
        // splits named, the model's choice marked):
        //   28 tiles, K 2048:  6 / 8* / 10 / 16: 13.9 / 13.2 / 15.3 / 15.0       32 tiles, K 8000: 4 / 8* / 16: 37.5 / 25.8 / 27.6
        //   96 tiles, K 8000:  2 / 3 / 4 / 5*: 68 / 84 / 66 / 58                 128 tiles, K 8000: 2 / 3 / 4* / 5: 81 / 86 / 72 / 79
        //   160 tiles, K 2048: 1 / 2 / 3* / 4: 36 / 38 / 29 / 32                 192 tiles, K 2048: 1 / 2 / 3 / 4*: 36 - 39 / 38 / 39 / 34
        //   224, 256 tiles, K 2048: 1* / 2: 36 / 38.5, 37 / 40                   256 tiles, K 8000: 1* / 2 / 4: 127 / 129 / 132
        //   320 tiles, K 2048: 1 / 2: 63.5 / 55.9 (3* by the model)              384 tiles, K 2048: 1 / 2* / 3: 63.6 / 58.5 / 70.8
        //   384 tiles, K 8000: 1 / 2*: 231 / 193                                 512 tiles, K 2048: 1* / 2: 67 / 75
        //   500 and 625 tiles, K 2048: unsplit faster than split in two (no split is considered from 512 tiles on)
        splits = 1;
        if (tiles < 2 * kNumCU) {
            const int ktiles = (K + bk - 1) / bk;
            const double per_split = (double)M * N * batch * 1.14e-4;
            auto cost = [&](int sp) {
                const int64_t rounds = (tiles * sp + kNumCU - 1) / kNumCU;
                const int steps = (ktiles + sp - 1) / sp * bk;
                double c = (double)rounds * steps;
                if (rounds == 1 && steps < 6000) c *= 1.2;
                if (sp > 1) c += 340.0 + sp * per_split;
                return c;
            };
            int smax = K / (16 * bk);
            if (smax > 16) smax = 16;
            double best = cost(1);
            for (int sp = 2; sp <= smax; ++sp) {
                const double c = cost(sp);
                if (c < 0.95 * best) { best = c; splits = sp; }
            }
        }
    }
    // contraction elements per split, rounded up to the k tile; drop empty trailing splits
    int kper = ((K + splits - 1) / splits + bk - 1) / bk * bk;
    if (kper < bk) kper = bk;
    splits = (K + kper - 1) / kper;
    if (splits < 1) splits = 1;
    pl.splits = splits;
    return pl;
}

int64_t gemm_ws_floats(int M, int N, int K, int batch, int force_cfg, int force_splits) {
    const GemmPlan pl = gemm_plan(M, N, K, batch, force_cfg, force_splits);
    int splits = pl.splits;
    if (cfg_dma_only(pl.cfg)) {      // direct-to-LDS only: also cover what runs if the operands rule it out
        const GemmPlan fb = gemm_plan(M, N, K, batch, CFG_64_REG, force_splits);
        if (fb.splits > splits) splits = fb.splits;
    }
    return splits > 1 ? (int64_t)splits * batch * M * N : 0;
}

static bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

// May the direct-to-LDS kernel run this problem?  Its loads are unmasked 16-byte loads.
static bool dma_eligible(const GemmDesc& d, const GemmKParams& p) {
    if (!p.vecA || !p.vecB) return false;
    if (d.K < kDmaBK || p.kper % kDmaBK != 0) return false;      // (a contraction tail of fewer than 16 steps is handled)
    if (!d.a_kc && (p.Mr < 4 || p.Mr % 4 != 0 || p.Mr > d.lda)) return false;
    if (!d.b_kc && (p.Nr < 4 || p.Nr % 4 != 0 || p.Nr > d.ldb)) return false;
    const int64_t lim = (int64_t)1 << 29;      // per-lane offsets are 32-bit byte offsets
    if ((d.a_kc ? (int64_t)d.M * d.lda : kDmaBK * d.lda + d.M) >= lim) return false;
    if ((d.b_kc ? (int64_t)d.N * d.ldb : kDmaBK * d.ldb + d.N) >= lim) return false;
    return true;
}

static void launch_dma(int cfg, const GemmKParams& p, bool a_kc, bool b_kc, dim3 grid, hipStream_t s) {
    if (cfg == CFG_128x64 || cfg == CFG_64x128 || cfg == CFG_128) launch_dma128(cfg, p, a_kc, b_kc, grid, s);
    else launch_dma64(cfg, p, a_kc, b_kc, grid, s);
}

static GemmKParams fill_params(const GemmDesc& d, const GemmPlan& pl, float* ws) {
    GemmKParams p;
    p.A = d.A; p.lda = d.lda; p.a_bstride = d.a_bstride;
    p.B = d.B; p.ldb = d.ldb; p.b_bstride = d.b_bstride;
    p.C = d.C; p.ldc = d.ldc; p.c_bstride = d.c_bstride;
    p.M = d.M; p.N = d.N; p.K = d.K; p.batch = d.batch;
    p.Mr = d.a_pad4 ? (d.M + 3) / 4 * 4 : d.M;
    p.Nr = d.b_pad4 ? (d.N + 3) / 4 * 4 : d.N;
    p.splits = pl.splits;
    const int bk = kCfgs[pl.cfg].bk;
    int kper = ((d.K + pl.splits - 1) / pl.splits + bk - 1) / bk * bk;
    if (kper < bk) kper = bk;
    p.kper = kper;
    p.tiles_m = (d.M + pl.bm - 1) / pl.bm;
    p.tiles_n = (d.N + pl.bn - 1) / pl.bn;
    p.vecA = aligned16(d.A) && (d.lda % 4 == 0) && (d.a_bstride % 4 == 0);
    p.vecB = aligned16(d.B) && (d.ldb % 4 == 0) && (d.b_bstride % 4 == 0);
    p.ws = ws;
    p.epi = d.epi;
    return p;
}

int gemm_launch(const GemmDesc& d, float* ws, int64_t ws_floats, hipStream_t stream) {
    if (d.M <= 0 || d.N <= 0 || d.batch <= 0) return 0;
    if (d.epi.rowsum_dst != nullptr && d.a_kc) return note_hip_error(hipErrorInvalidValue);
    // fused row sums and the side sum are the work of the kernel that owns a whole tile: unsplit, not the in-workgroup split
    const bool rowsum = d.epi.rowsum_dst != nullptr || d.epi.side_sum_src != nullptr;
    GemmPlan pl = gemm_plan(d.M, d.N, d.K, d.batch, d.force_cfg, rowsum ? 1 : d.force_splits);
    GemmKParams p = fill_params(d, pl, ws);
    const bool kg_cfg = cfg_kg(pl.cfg);
    if (cfg_dma_only(pl.cfg) &&
        !(dma_eligible(d, p) && (!kg_cfg || (!rowsum && d.K / (pl.cfg == CFG_KG_32x64 ? kKgWideBK : kDmaBK) >= kKGroups)))) {
        pl = gemm_plan(d.M, d.N, d.K, d.batch, CFG_64_REG, rowsum ? 1 : d.force_splits);
        p = fill_params(d, pl, ws);
    }
    if (d.force_cfg < 0 && pl.splits == 1 && !dma_eligible(d, p)) {
        // a large problem the direct-to-LDS kernel cannot take (ragged contraction, unaligned rows): among the
        // register-staged kernels the 128x128 tile with 8 wavefronts is the fastest from about 3000 64x64 tiles on
        const int64_t t64 = (int64_t)p.tiles_m * p.tiles_n * d.batch;
        if (t64 >= 3072 && d.M >= 512 && d.N >= 512) {
            pl = gemm_plan(d.M, d.N, d.K, d.batch, CFG_128_REG, 1);
            p = fill_params(d, pl, ws);
        }
    }
    if (pl.splits > 1 && (ws == nullptr || ws_floats < (int64_t)pl.splits * d.batch * d.M * d.N)) return note_hip_error(hipErrorInvalidValue);
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)(d.batch * pl.splits));
    if (cfg_kg(pl.cfg)) {      // (the plan may have been replaced above)
        launch_kg(pl.cfg, p, d.a_kc, d.b_kc, grid, stream);
    } else if ((pl.cfg == CFG_64 || pl.cfg >= CFG_128x64) && dma_eligible(d, p)) launch_dma(pl.cfg, p, d.a_kc, d.b_kc, grid, stream);
    else launch_legacy(pl.cfg == CFG_128_REG, p, d.a_kc, d.b_kc, grid, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return note_hip_error(e);
    if (pl.splits > 1) {
        // one float4 per thread when rows are multiples of 4 long, else one element per thread
        const int64_t work = (d.N & 3) == 0 ? (int64_t)d.M * d.N / 4 : (int64_t)d.M * d.N;
        int64_t gx = (work + 255) / 256;
        if (gx > 4096) gx = 4096;
        if (gx < 1) gx = 1;
        hipLaunchKernelGGL(gemm_reduce_kernel, dim3((unsigned)gx, (unsigned)d.batch), dim3(256), 0, stream, p);
        e = hipGetLastError();
    }
    return note_hip_error(e);
}

// Thin products X R^T in one launch (see gemm_thin_grouped_kernel); a problem that kernel cannot take is launched by
// itself, unsplit.
static int gemm_launch_grouped_thin(const GemmDesc* d, int count, hipStream_t stream) {
    ThinGroupParams gp;
    gp.ngroups = 0;
    int tiles = 0, batch = 0;
    auto flush = [&]() -> int {
        if (gp.ngroups == 0) return 0;
        gp.tile_start[gp.ngroups] = tiles;
        launch_thin(gp, dim3((unsigned)tiles, 1, (unsigned)batch), stream);
        gp.ngroups = 0;
        tiles = 0;
        const hipError_t e = hipGetLastError();
        return e == hipSuccess ? 0 : note_hip_error(e);
    };
    for (int i = 0; i < count; ++i) {
        const GemmDesc& di = d[i];
        if (di.M <= 0 || di.N <= 0 || di.batch <= 0) continue;
        if (!di.a_kc || !di.b_kc || di.batch != d[0].batch || di.epi.kind != EPI_STORE || di.epi.rowsum_dst != nullptr)
            return note_hip_error(hipErrorInvalidValue);
        const GemmPlan pl = gemm_plan(di.M, di.N, di.K, di.batch, CFG_KG_32x32, 1);
        const GemmKParams q = fill_params(di, pl, nullptr);
        if (!dma_eligible(di, q) || di.K / kDmaBK < kThinKGroups) {
            GemmDesc one = di;
            one.force_cfg = -1; one.force_splits = 1;
            if (gemm_launch(one, nullptr, 0, stream) != 0) return -1;
            continue;
        }
        batch = di.batch;
        ThinProblem& t = gp.g[gp.ngroups];
        t.A = di.A; t.B = di.B; t.C = di.C;
        t.lda = di.lda; t.ldb = di.ldb; t.ldc = di.ldc;
        t.a_bstride = di.a_bstride; t.b_bstride = di.b_bstride; t.c_bstride = di.c_bstride;
        t.M = di.M; t.N = di.N; t.K = di.K;
        gp.tile_start[gp.ngroups] = tiles;
        tiles += q.tiles_m * q.tiles_n;
        if (++gp.ngroups == kMaxThin && flush() != 0) return -1;
    }
    return flush();
}

int gemm_launch_grouped(const GemmDesc* d, int count, hipStream_t stream, bool thin) {
    if (thin) return gemm_launch_grouped_thin(d, count, stream);
    // Two passes over the problems: those the direct-to-LDS kernel accepts, then the rest (ragged or unaligned
    // ones, e.g. a layer whose width is not a multiple of 4) with the register-staged kernel.
    for (int pass = 0; pass < 2; ++pass) {
        const bool dma = pass == 0;
        GemmGroupParams gp;
        gp.ngroups = 0;
        int tiles = 0, batch = 0;
        bool a_kc = false, b_kc = false;
        auto flush = [&]() -> int {
            if (gp.ngroups == 0) return 0;
            gp.tile_start[gp.ngroups] = tiles;
            const dim3 grid((unsigned)tiles, 1, (unsigned)batch);
            if (dma) launch_grouped_dma(gp, a_kc, b_kc, grid, stream);
            else launch_grouped_legacy(gp, a_kc, b_kc, grid, stream);
            gp.ngroups = 0;
            tiles = 0;
            const hipError_t e = hipGetLastError();
            return e == hipSuccess ? 0 : note_hip_error(e);
        };
        for (int i = 0; i < count; ++i) {
            const GemmDesc& di = d[i];
            if (di.M <= 0 || di.N <= 0 || di.batch <= 0) continue;
            if (di.a_kc != d[0].a_kc || di.b_kc != d[0].b_kc || di.batch != d[0].batch) return note_hip_error(hipErrorInvalidValue);
            if (di.epi.rowsum_dst != nullptr && di.a_kc) return note_hip_error(hipErrorInvalidValue);
            const GemmPlan pl = gemm_plan(di.M, di.N, di.K, di.batch, CFG_64, 1);      // 64x64 tiles, unsplit
            const GemmKParams q = fill_params(di, pl, nullptr);
            if (dma_eligible(di, q) != dma) continue;
            a_kc = di.a_kc; b_kc = di.b_kc; batch = di.batch;
            gp.g[gp.ngroups] = q;
            gp.tile_start[gp.ngroups] = tiles;
            tiles += q.tiles_m * q.tiles_n;
            if (++gp.ngroups == kMaxGroups && flush() != 0) return -1;
        }
        if (flush() != 0) return -1;
    }
    return 0;
}

}  // namespace mavg

static thread_local hipError_t g_last_error = hipSuccess;
namespace mavg {
int note_hip_error(hipError_t e) {
    if (e != hipSuccess) g_last_error = e;
    return (int)e;
}
}  // namespace mavg

extern "C" const char* mavg_last_error(void) { return hipGetErrorString(g_last_error); }

// ---- exported test/tuning entry points -----------------------------------------------------------
using namespace mavg;

extern "C" int64_t mavg_gemm_workspace_bytes(int32_t m, int32_t n, int32_t k, int32_t cfg, int32_t splits) {
    if (m < 1 || n < 1 || k < 0) return MAVG_E_DIM;
    if (cfg >= kNumCfgs || splits < 0) return MAVG_E_FLAG;
    return gemm_ws_floats(m, n, k, 1, cfg, splits) * 4 + 256;
}

extern "C" int32_t mavg_gemm(const float* a, int64_t lda, int32_t a_kc, const float* b, int64_t ldb, int32_t b_kc,
                             float* c, int64_t ldc, int32_t m, int32_t n, int32_t k, int32_t epi, const float* bias,
                             const float* aux, int64_t ldaux, float alpha, float beta, int32_t cfg, int32_t splits,
                             void* workspace, int64_t workspace_bytes, void* stream) {
    if (!a || !b || !c) return MAVG_E_NULL;
    if (m < 1 || n < 1 || k < 0) return MAVG_E_DIM;
    if (cfg >= kNumCfgs || splits < 0 || epi < EPI_STORE || epi > EPI_AXPBY) return MAVG_E_FLAG;
    if ((epi == EPI_BIAS || epi == EPI_BIAS_SIGMOID) && !bias) return MAVG_E_NULL;
    if (epi == EPI_MUL_DSIGMOID && !aux) return MAVG_E_NULL;
    if (lda < (a_kc ? k : m) || ldb < (b_kc ? k : n) || ldc < n || (epi == EPI_MUL_DSIGMOID && ldaux < n)) return MAVG_E_ALIGN;
    const int64_t need = gemm_ws_floats(m, n, k, 1, cfg, splits);
    if (need > 0 && (!workspace || workspace_bytes < need * 4 + 256)) return MAVG_E_WORKSPACE;
    GemmDesc g;
    g.A = a; g.lda = lda; g.a_kc = a_kc != 0;
    g.B = b; g.ldb = ldb; g.b_kc = b_kc != 0;
    g.C = c; g.ldc = ldc;
    g.M = m; g.N = n; g.K = k;
    g.epi.kind = epi; g.epi.bias = bias; g.epi.aux = aux; g.epi.ldaux = ldaux; g.epi.alpha = alpha; g.epi.beta = beta;
    g.force_cfg = cfg; g.force_splits = splits;
    float* ws = workspace ? reinterpret_cast<float*>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~uintptr_t(255)) : nullptr;
    return gemm_launch(g, ws, need, static_cast<hipStream_t>(stream)) == 0 ? MAVG_OK : MAVG_E_LAUNCH;
}

extern "C" int32_t mavg_gemm_grouped(const mavg_gemm_problem* pr, int32_t count, int32_t a_kc, int32_t b_kc, void* stream) {
    if (!pr) return MAVG_E_NULL;
    if (count < 1 || count > kMaxGroups) return MAVG_E_DIM;
    GemmDesc g[kMaxGroups];
    for (int i = 0; i < count; ++i) {
        const mavg_gemm_problem& q = pr[i];
        if (!q.a || !q.b || !q.c) return MAVG_E_NULL;
        if (q.m < 1 || q.n < 1 || q.k < 0) return MAVG_E_DIM;
        if (q.epi < EPI_STORE || q.epi > EPI_AXPBY) return MAVG_E_FLAG;
        if ((q.epi == EPI_BIAS || q.epi == EPI_BIAS_SIGMOID) && !q.bias) return MAVG_E_NULL;
        if (q.epi == EPI_MUL_DSIGMOID && !q.aux) return MAVG_E_NULL;
        if (q.rowsum_dst && a_kc) return MAVG_E_FLAG;
        if (q.lda < (a_kc ? q.k : q.m) || q.ldb < (b_kc ? q.k : q.n) || q.ldc < q.n || (q.epi == EPI_MUL_DSIGMOID && q.ldaux < q.n))
            return MAVG_E_ALIGN;
        GemmDesc& d = g[i];
        d.A = q.a; d.lda = q.lda; d.a_kc = a_kc != 0;
        d.B = q.b; d.ldb = q.ldb; d.b_kc = b_kc != 0;
        d.C = q.c; d.ldc = q.ldc;
        d.M = q.m; d.N = q.n; d.K = q.k;
        d.a_pad4 = q.a_pad4 != 0; d.b_pad4 = q.b_pad4 != 0;
        d.epi.kind = q.epi; d.epi.bias = q.bias; d.epi.aux = q.aux; d.epi.ldaux = q.ldaux; d.epi.alpha = q.alpha; d.epi.beta = q.beta;
        d.epi.rowsum_dst = q.rowsum_dst; d.epi.rowsum_alpha = q.rowsum_alpha; d.epi.rowsum_beta = q.rowsum_beta;
    }
    return gemm_launch_grouped(g, count, static_cast<hipStream_t>(stream)) == 0 ? MAVG_OK : MAVG_E_LAUNCH;
}
