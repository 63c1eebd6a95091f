// Device side of the fp32 MFMA GEMM: kernel parameters, epilogues, tile order, the register-staged and the
// direct-to-LDS kernel bodies.  Included by the translation units that instantiate the kernels (one per kernel
// family, so that they compile in parallel); everything here is a template or forced inline.
#pragma once
#include "gemm.h"
#include "../../include/mavg.h"
#include "device_math.h"
#include <cstddef>
#include <utility>
#include <type_traits>

namespace mavg {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
// Used wherever the accumulator arrays are indexed, so that every index is a constant from the start
// and the accumulators stay in registers.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

struct GemmKParams {
    const float* A; int64_t lda, a_bstride;
    const float* B; int64_t ldb, b_bstride;
    float* C; int64_t ldc, c_bstride;
    int M, N, K, batch, splits, kper;   // kper: contraction elements per split (multiple of the k tile)
    int Mr, Nr;                         // readable extents of m/n-contiguous operands (M, N or those rounded up to 4)
    int tiles_m, tiles_n;
    int vecA, vecB;                     // operands may be read with 16-byte loads
    float* ws;                          // partial sums [batch][split][M][N] when splits > 1
    Epilogue epi;
};

// ---- epilogue ------------------------------------------------------------------------------------

struct EpiCtx {       // per-batch resolved pointers and scalars
    const float* bias; const float* aux; float* C; float* C2; const float* rowvec; float alpha; float* lastcol_dst;
};

__device__ __forceinline__ EpiCtx epi_ctx(const Epilogue& e, float* C, int64_t c_bstride, int b) {
    EpiCtx c;
    c.bias = e.bias ? e.bias + (int64_t)b * e.bias_bstride : nullptr;
    c.aux = e.aux ? e.aux + (int64_t)b * e.aux_bstride : nullptr;
    c.C = C ? C + (int64_t)b * c_bstride : nullptr;
    c.C2 = e.C2 ? e.C2 + (int64_t)b * e.c2_bstride : nullptr;
    c.rowvec = e.rowvec ? e.rowvec + (int64_t)b * e.rowvec_bstride : nullptr;
    c.lastcol_dst = e.lastcol_dst ? e.lastcol_dst + (int64_t)b * e.lastcol_bstride : nullptr;
    c.alpha = e.alpha;
    if (e.alpha_dev0) c.alpha *= e.alpha_dev0[b];
    if (e.alpha_dev1) c.alpha *= e.alpha_dev1[b];
    return c;
}

template <int KIND>
__device__ __forceinline__ void epi_apply(const Epilogue& e, const EpiCtx& c, int64_t ldc, int N, int m, int n, float v) {
    if (KIND == EPI_STORE) {
        c.C[(int64_t)m * ldc + n] = v;
    } else if (KIND == EPI_BIAS) {
        c.C[(int64_t)m * ldc + n] = v + c.bias[n];
    } else if (KIND == EPI_BIAS_SIGMOID) {
        c.C[(int64_t)m * ldc + n] = c.alpha * (e.act_tanh ? tanhf(v + c.bias[n]) : sigmoidf_dev(v + c.bias[n]));
    } else if (KIND == EPI_MUL_DSIGMOID) {
        const float a = c.aux[(int64_t)m * e.ldaux + n];
        c.C[(int64_t)m * ldc + n] = e.act_tanh ? v * (1.f - a * a) : v * a * (1.f - a);
    } else if (KIND == EPI_AXPBY) {
        float* dst = (c.lastcol_dst && n == e.lastcol) ? c.lastcol_dst + m : c.C + (int64_t)m * ldc + n;
        float r = c.alpha * v;
        if (e.beta != 0.f) r += e.beta * *dst;
        *dst = r;
        if (c.C2) { const int64_t j = (int64_t)m * e.ldc2 + n; c.C2[j] += r; }
    } else if (KIND == EPI_BIAS_SIGMOID_SAMPLE) {
        const float p = sigmoidf_dev(v + c.bias[n]);
        if (c.C) c.C[(int64_t)m * ldc + n] = p;
        const float u = philox_uniform((uint64_t)m * (uint64_t)N + (uint64_t)n, e.key0, e.key1, e.step, e.layer, e.phase);
        c.C2[(int64_t)m * e.ldc2 + n] = (u < p) ? 1.f : 0.f;
    } else if (KIND == EPI_ROWSCALE_ADD) {
        c.C[(int64_t)m * ldc + n] = c.alpha * v + c.rowvec[m] * c.aux[(int64_t)m * e.ldaux + n];
    }
}

// The side sum of an epilogue (see gemm.h), by a whole workgroup of at least 256 threads; `sh`: 4 floats of LDS
// that nothing else uses any more.  Fixed order: thread t of the first 256 adds elements t, t + 256, ..., a wavefront
// adds its lanes by butterfly, the four wavefronts' sums are added pairwise.
__device__ __forceinline__ void side_sum(const Epilogue& e, float* sh) {
    __syncthreads();
    const int tid = threadIdx.x;
    float s = 0.f;
    if (tid < 256)
        for (int i = tid; i < e.side_sum_n; i += 256) s += e.side_sum_src[i];
    s = wave_sum(s);
    if (tid < 256 && (tid & 63) == 0) sh[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) *e.side_sum_dst = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// Element at byte offset `off` from a pointer that is uniform over the wavefront: the form the hardware addresses
// as scalar base + 32-bit per-lane offset, which costs one vector register per access pattern instead of a
// 64-bit address per access.
__device__ __forceinline__ float* at_off(float* ubase, uint32_t off) {
    return reinterpret_cast<float*>(reinterpret_cast<char*>(ubase) + off);
}
__device__ __forceinline__ const float* at_off(const float* ubase, uint32_t off) {
    return reinterpret_cast<const float*>(reinterpret_cast<const char*>(ubase) + off);
}

// Write a wavefront's accumulators through epilogue KIND.  Accumulator element v of a lane sits at
// row 8*(v/4) + 4*(lane/32) + v%4, column lane%32 of its 32x32 block.  `mbase` is uniform over the wavefront.
// Every access is (uniform row pointer) + (per-lane byte offset): row 8*(v/4) + v%4 of the block goes into the
// scalar pointer, the lane's 4*(lane/32) rows and its column into one offset register per matrix.
// `band` (uniform over the wavefront): -1 = all 16 elements; 0..3 = only elements 4 band .. 4 band + 3, i.e. rows
// 8 band .. 8 band + 7 of each 32x32 block (a workgroup whose wavefronts share the epilogue of one accumulator).
template <int KIND, int TM, int TN>
__device__ __forceinline__ void write_tile(const floatx16 (&acc)[TM][TN], const Epilogue& e, const EpiCtx& c,
                                           int64_t ldc, int M, int N, int mbase, int nbase, int lrow, int lcol, int band = -1) {
    constexpr bool kReadsC = KIND == EPI_AXPBY;
    constexpr bool kReadsAux = KIND == EPI_MUL_DSIGMOID || KIND == EPI_ROWSCALE_ADD;
    constexpr bool kBias = KIND == EPI_BIAS || KIND == EPI_BIAS_SIGMOID || KIND == EPI_BIAS_SIGMOID_SAMPLE;
    const int mb = __builtin_amdgcn_readfirstlane(mbase);
    static_for<TM * TN>([&](auto bc) {
        constexpr int t = decltype(bc)::value;
        constexpr int i = t / TN, j = t % TN;
        // Does this 32-column block hold the column that goes to a separate vector (uniform over the wavefront)?
        // Only then do the accesses need a per-lane choice of destination.
        bool has_lastcol = false;
        if constexpr (KIND == EPI_AXPBY)
            has_lastcol = c.lastcol_dst != nullptr && e.lastcol >= nbase + j * 32 && e.lastcol < nbase + j * 32 + 32;
        // A block that lies wholly inside the matrix needs no per-element bounds checks (uniform over the wavefront).
        const bool interior = mb + i * 32 + 32 <= M && nbase + j * 32 + 32 <= N;
        auto block = [&](auto lcc, auto inc) {
            constexpr bool LC = decltype(lcc)::value, IN = decltype(inc)::value;
            const int n = nbase + j * 32 + lcol;
            const bool n_ok = IN || n < N;
            const uint32_t offC = (uint32_t)(((int64_t)(4 * lrow) * ldc + n) * 4);
            const uint32_t offAux = kReadsAux ? (uint32_t)(((int64_t)(4 * lrow) * e.ldaux + n) * 4) : 0u;
            const uint32_t offC2 = (KIND == EPI_AXPBY || KIND == EPI_BIAS_SIGMOID_SAMPLE) ? (uint32_t)(((int64_t)(4 * lrow) * e.ldc2 + n) * 4) : 0u;
            const bool lastcol = LC && n == e.lastcol;
            float bias_n = 0.f;
            if (kBias && n_ok) bias_n = c.bias[n];
            float old[16];
            if constexpr (kReadsC || kReadsAux) {
                // read-modify-write epilogues: issue the 16 loads of a 32x32 block back to back, then combine and
                // store, so that their latencies overlap instead of adding up
                const bool need_old = kReadsAux || e.beta != 0.f;
                static_for<16>([&](auto vc) {
                    constexpr int v = decltype(vc)::value;
                    const int mu = mb + i * 32 + 8 * (v >> 2) + (v & 3);
                    const int m = mu + 4 * lrow;
                    old[v] = 0.f;
                    if (need_old && (band < 0 || band == (v >> 2)) && (IN || m < M) && n_ok) {
                        if constexpr (kReadsC) old[v] = lastcol ? c.lastcol_dst[m] : *at_off(c.C + (int64_t)mu * ldc, offC);
                        else old[v] = *at_off(c.aux + (int64_t)mu * e.ldaux, offAux);
                    }
                });
            }
            static_for<16>([&](auto vc) {
                constexpr int v = decltype(vc)::value;
                const int mu = mb + i * 32 + 8 * (v >> 2) + (v & 3);
                const int m = mu + 4 * lrow;
                if ((band < 0 || band == (v >> 2)) && (IN || m < M) && n_ok) {
                    const float a = acc[i][j][v];
                    float* dst = at_off(c.C + (int64_t)mu * ldc, offC);
                    if constexpr (KIND == EPI_STORE) {
                        *dst = a;
                    } else if constexpr (KIND == EPI_BIAS) {
                        *dst = a + bias_n;
                    } else if constexpr (KIND == EPI_BIAS_SIGMOID) {
                        *dst = c.alpha * (e.act_tanh ? tanhf(a + bias_n) : sigmoidf_dev(a + bias_n));
                    } else if constexpr (KIND == EPI_MUL_DSIGMOID) {
                        *dst = e.act_tanh ? a * (1.f - old[v] * old[v]) : a * old[v] * (1.f - old[v]);
                    } else if constexpr (KIND == EPI_AXPBY) {
                        const float r = c.alpha * a + e.beta * old[v];
                        if (lastcol) c.lastcol_dst[m] = r;
                        else *dst = r;
                        if (c.C2) *at_off(c.C2 + (int64_t)mu * e.ldc2, offC2) += r;
                    } else if constexpr (KIND == EPI_BIAS_SIGMOID_SAMPLE) {
                        const float pr = sigmoidf_dev(a + bias_n);
                        if (c.C) *dst = pr;
                        const float u = philox_uniform((uint64_t)m * (uint64_t)N + (uint64_t)n, e.key0, e.key1, e.step, e.layer, e.phase);
                        *at_off(c.C2 + (int64_t)mu * e.ldc2, offC2) = (u < pr) ? 1.f : 0.f;
                    } else {      // EPI_ROWSCALE_ADD
                        *dst = c.alpha * a + c.rowvec[m] * old[v];
                    }
                }
            });
        };
        if (has_lastcol) {
            if constexpr (KIND == EPI_AXPBY) block(std::true_type{}, std::false_type{});
        } else if (interior) {
            block(std::false_type{}, std::true_type{});
        } else {
            block(std::false_type{}, std::false_type{});
        }
    });
}

// Apply epilogue `kind` to four consecutive elements of a row (the split-contraction reducer).
template <int KIND>
__device__ __forceinline__ void epi_apply4(const Epilogue& e, const EpiCtx& c, int64_t ldc, int N, int m, int n, float4 s) {
    epi_apply<KIND>(e, c, ldc, N, m, n + 0, s.x);
    epi_apply<KIND>(e, c, ldc, N, m, n + 1, s.y);
    epi_apply<KIND>(e, c, ldc, N, m, n + 2, s.z);
    epi_apply<KIND>(e, c, ldc, N, m, n + 3, s.w);
}

#define MAVG_EPI_DISPATCH(kind, CALL)                                              \
    switch (kind) {                                                                \
    case EPI_STORE: { constexpr int KIND = EPI_STORE; CALL; break; }               \
    case EPI_BIAS: { constexpr int KIND = EPI_BIAS; CALL; break; }                 \
    case EPI_BIAS_SIGMOID: { constexpr int KIND = EPI_BIAS_SIGMOID; CALL; break; } \
    case EPI_MUL_DSIGMOID: { constexpr int KIND = EPI_MUL_DSIGMOID; CALL; break; } \
    case EPI_AXPBY: { constexpr int KIND = EPI_AXPBY; CALL; break; }               \
    case EPI_BIAS_SIGMOID_SAMPLE: { constexpr int KIND = EPI_BIAS_SIGMOID_SAMPLE; CALL; break; } \
    case EPI_ROWSCALE_ADD: { constexpr int KIND = EPI_ROWSCALE_ADD; CALL; break; } \
    default: break;                                                                \
    }

// ---- main kernel ---------------------------------------------------------------------------------

constexpr int kPad = 4;

// XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so the
// workgroups with equal (id mod 8) share an L2.  Each XCD gets one contiguous run of the tile sequence, which
// walks fastest along the smaller operand: that one is re-read for every tile of the run and has to stay in
// L2 (activations when M <= N, e.g. 256 x 8000; the other way round for a weight gradient), while a tile of
// the larger operand crosses the fabric once instead of once per XCD (measured on the 256 x 8000 x 2048
// layer: L2 fetch traffic 284 MB -> 85 MB).
__device__ __forceinline__ void tile_coords(const GemmKParams& p, int tile, int& tm_i, int& tn_i) {
    const int ntiles = p.tiles_m * p.tiles_n;
    const int xcd = tile % kNumXCD, slot = tile / kNumXCD;
    const int tq = ntiles / kNumXCD, tr = ntiles % kNumXCD;
    const int seq = xcd * tq + min(xcd, tr) + slot;          // bijection of [0, ntiles)
    if (p.M <= p.N) { tn_i = seq / p.tiles_m; tm_i = seq - tn_i * p.tiles_m; }
    else { tm_i = seq / p.tiles_n; tn_i = seq - tm_i * p.tiles_n; }
}


// Global -> register load of one operand tile (BR rows of the non-contracted index by BK contraction
// steps), zero-filled outside [0,R) x [k0,kend).  KC: the contraction index is the contiguous one.
template <bool GUARD, bool KC, int NLD, int BR, int BK, int NT>
__device__ __forceinline__ void load_operand(const float* __restrict__ P, int64_t ld, int vec, int r0, int R,
                                             int k0, int kend, int tid, float4 (&reg)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int f = tid + i * NT;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!GUARD) {      // tile fully inside the matrix, 16-byte aligned: one vector load, no checks
            if (KC) {
                const int r = f / (BK / 4), kq = f % (BK / 4);
                v = *reinterpret_cast<const float4*>(P + (int64_t)(r0 + r) * ld + (k0 + kq * 4));
            } else {
                const int k = f / (BR / 4), rq = f % (BR / 4);
                v = *reinterpret_cast<const float4*>(P + (int64_t)(k0 + k) * ld + (r0 + rq * 4));
            }
        } else if (KC) {
            const int r = f / (BK / 4), kq = f % (BK / 4);
            const int gr = r0 + r, gk = k0 + kq * 4;
            if (gr < R && gk < kend) {
                const float* src = P + (int64_t)gr * ld + gk;
                if (vec && gk + 3 < kend) v = *reinterpret_cast<const float4*>(src);
                else {
                    v.x = src[0];
                    if (gk + 1 < kend) v.y = src[1];
                    if (gk + 2 < kend) v.z = src[2];
                    if (gk + 3 < kend) v.w = src[3];
                }
            }
        } else {
            const int k = f / (BR / 4), rq = f % (BR / 4);
            const int gk = k0 + k, gr = r0 + rq * 4;
            if (gk < kend && gr < R) {
                const float* src = P + (int64_t)gk * ld + gr;
                if (vec && gr + 3 < R) v = *reinterpret_cast<const float4*>(src);
                else {
                    v.x = src[0];
                    if (gr + 1 < R) v.y = src[1];
                    if (gr + 2 < R) v.z = src[2];
                    if (gr + 3 < R) v.w = src[3];
                }
            }
        }
        reg[i] = v;
    }
}

// Register -> LDS store of the tile, k-major: S[k][r].
template <bool KC, int NLD, int BR, int BK, int LDS_LD, int NT>
__device__ __forceinline__ void store_operand(float* S, int tid, const float4 (&reg)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int f = tid + i * NT;
        if (KC) {
            const int r = f / (BK / 4), kq = f % (BK / 4);
            S[(kq * 4 + 0) * LDS_LD + r] = reg[i].x;
            S[(kq * 4 + 1) * LDS_LD + r] = reg[i].y;
            S[(kq * 4 + 2) * LDS_LD + r] = reg[i].z;
            S[(kq * 4 + 3) * LDS_LD + r] = reg[i].w;
        } else {
            const int k = f / (BR / 4), rq = f % (BR / 4);
            *reinterpret_cast<float4*>(&S[k * LDS_LD + rq * 4]) = reg[i];
        }
    }
}

// BM x BN output tile, BK contraction steps per LDS stage, WM x WN wavefronts (64*WM*WN threads); each
// wavefront owns (BM/WM) x (BN/WN) as TM x TN accumulators of 32x32.
template <int BM, int BN, int BK, int WM, int WN, int PF, bool AKC, bool BKC>
__device__ __forceinline__ void gemm_body(const GemmKParams& p, const int tile, const int bz) {
    static_assert(PF >= 2 && PF % 2 == 0, "prefetch depth must be even");
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int LDAS = BM + kPad, LDBS = BN + kPad;
    constexpr int A_LD = BM * BK / 4 / NT, B_LD = BN * BK / 4 / NT;   // float4 loads per thread per tile
    static_assert(TM >= 1 && TN >= 1 && BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "bad wavefront grid");
    static_assert(A_LD >= 1 && B_LD >= 1 && A_LD * NT * 4 == BM * BK && B_LD * NT * 4 == BN * BK, "tile does not divide over the threads");
    static_assert(BM <= NT, "row sums need one thread per tile row");
    __shared__ __attribute__((aligned(16))) float As[2][BK][LDAS];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][LDBS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave / WN) * (BM / WM), wn = (wave % WN) * (BN / WN);
    const int b = bz / p.splits, split = bz - b * p.splits;
    int tm_i, tn_i;
    tile_coords(p, tile, tm_i, tn_i);
    const int m0 = tm_i * BM, n0 = tn_i * BN;
    const int kbeg = split * p.kper;
    const int kend = min(p.K, kbeg + p.kper);
    const float* __restrict__ A = p.A + (int64_t)b * p.a_bstride;
    const float* __restrict__ B = p.B + (int64_t)b * p.b_bstride;

    floatx16 acc[TM][TN];
    static_for<TM * TN>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        acc[t / TN][t % TN] = floatx16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    });

    const int nkt = (kend - kbeg + BK - 1) / BK;
    const int lrow = lane >> 5, lcol = lane & 31;
    // optional fused row sums of the A operand (sum over the contraction index), e.g. the bias gradient
    // delta^T 1 next to the weight gradient delta^T A: taken from the LDS tiles by the first tile column only
    const bool do_rowsum = !AKC && p.epi.rowsum_dst != nullptr && tn_i == 0 && tid < BM;
    float rowsum = 0.f;
    const float* __restrict__ rw = p.epi.rowsum_w ? p.epi.rowsum_w + (int64_t)b * p.epi.rowsum_w_bstride + kbeg : nullptr;

    // The loop over k-tiles.  Global loads run PF tiles ahead of the multiply: tile kt+PF is requested while
    // tile kt is multiplied out of LDS, and lives in registers until it is copied to the other LDS buffer
    // one iteration before its turn.  A workgroup that is alone on its compute unit (the skinny
    // minibatch-256 shapes) needs that many bytes in flight to cover HBM latency.  Inside a tile the MFMA
    // operands of step kk+2 are read from LDS while step kk is issued.
    auto mainloop = [&](auto guard_c) {
        constexpr bool GUARD = decltype(guard_c)::value;
        float4 ra[PF][A_LD], rb[PF][B_LD];
        static_for<PF>([&](auto sc) {
            constexpr int st = decltype(sc)::value;
            if (st < nkt) {
                load_operand<GUARD, AKC, A_LD, BM, BK, NT>(A, p.lda, p.vecA, m0, p.M, kbeg + st * BK, kend, tid, ra[st]);
                load_operand<GUARD, BKC, B_LD, BN, BK, NT>(B, p.ldb, p.vecB, n0, p.N, kbeg + st * BK, kend, tid, rb[st]);
            }
        });
        if (nkt > 0) {
            store_operand<AKC, A_LD, BM, BK, LDAS, NT>(&As[0][0][0], tid, ra[0]);
            store_operand<BKC, B_LD, BN, BK, LDBS, NT>(&Bs[0][0][0], tid, rb[0]);
        }
        __syncthreads();
        for (int kt0 = 0; kt0 < nkt; kt0 += PF) {
            static_for<PF>([&](auto sc) {
                constexpr int st = decltype(sc)::value;      // register slot of tile kt (PF is even: LDS buffer = st & 1)
                constexpr int buf = st & 1;
                const int kt = kt0 + st;
                if (kt < nkt) {
                    if (kt + PF < nkt) {                      // slot st was copied to LDS an iteration ago: refill it
                        load_operand<GUARD, AKC, A_LD, BM, BK, NT>(A, p.lda, p.vecA, m0, p.M, kbeg + (kt + PF) * BK, kend, tid, ra[st]);
                        load_operand<GUARD, BKC, B_LD, BN, BK, NT>(B, p.ldb, p.vecB, n0, p.N, kbeg + (kt + PF) * BK, kend, tid, rb[st]);
                    }
                    float fa[2][TM], fb[2][TN];
#pragma unroll
                    for (int i = 0; i < TM; ++i) fa[0][i] = As[buf][lrow][wm + i * 32 + lcol];
#pragma unroll
                    for (int j = 0; j < TN; ++j) fb[0][j] = Bs[buf][lrow][wn + j * 32 + lcol];
                    static_for<BK / 2>([&](auto kc) {
                        constexpr int ks = decltype(kc)::value;
                        constexpr int cur = ks & 1, nxt = cur ^ 1;
                        if constexpr (ks + 1 < BK / 2) {
#pragma unroll
                            for (int i = 0; i < TM; ++i) fa[nxt][i] = As[buf][2 * (ks + 1) + lrow][wm + i * 32 + lcol];
#pragma unroll
                            for (int j = 0; j < TN; ++j) fb[nxt][j] = Bs[buf][2 * (ks + 1) + lrow][wn + j * 32 + lcol];
                        }
                        static_for<TM * TN>([&](auto tc) {
                            constexpr int t = decltype(tc)::value;
                            constexpr int i = t / TN, j = t % TN;
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
                        });
                    });
                    if (do_rowsum) {
                        if (rw) {      // (tiles are zero-filled past kend; the weights are not read there)
#pragma unroll
                            for (int kk = 0; kk < BK; ++kk)
                                if (kbeg + kt * BK + kk < kend) rowsum += As[buf][kk][tid] * rw[kt * BK + kk];
                        } else {
#pragma unroll
                            for (int kk = 0; kk < BK; ++kk) rowsum += As[buf][kk][tid];
                        }
                    }
                    if (kt + 1 < nkt) {
                        constexpr int nx = (st + 1) % PF;
                        store_operand<AKC, A_LD, BM, BK, LDAS, NT>(&As[buf ^ 1][0][0], tid, ra[nx]);
                        store_operand<BKC, B_LD, BN, BK, LDBS, NT>(&Bs[buf ^ 1][0][0], tid, rb[nx]);
                    }
                    __syncthreads();
                }
            });
        }
    };
    const bool interior = p.vecA && p.vecB && m0 + BM <= p.M && n0 + BN <= p.N && ((kend - kbeg) % BK) == 0;
    if (interior) mainloop(std::false_type{});
    else mainloop(std::true_type{});

    if (do_rowsum && m0 + tid < p.M) {
        float* d = p.epi.rowsum_dst + (int64_t)b * p.epi.rowsum_bstride + m0 + tid;
        float r = p.epi.rowsum_alpha * rowsum;
        if (p.epi.alpha_dev0) r *= p.epi.alpha_dev0[b];
        if (p.epi.alpha_dev1) r *= p.epi.alpha_dev1[b];
        if (p.epi.rowsum_beta != 0.f) r += p.epi.rowsum_beta * *d;
        *d = r;
        if (p.epi.rowsum_dst2) p.epi.rowsum_dst2[(int64_t)b * p.epi.rowsum2_bstride + m0 + tid] += r;
    }
    if (p.splits > 1) {
        // split contraction: store the partial tile; gemm_reduce_kernel adds the partials in split order
        Epilogue raw;
        EpiCtx c;
        c.bias = nullptr; c.aux = nullptr; c.C2 = nullptr; c.rowvec = nullptr; c.alpha = 1.f; c.lastcol_dst = nullptr;
        c.C = p.ws + ((int64_t)bz * p.M) * p.N;
        write_tile<EPI_STORE, TM, TN>(acc, raw, c, p.N, p.M, p.N, m0 + wm, n0 + wn, lrow, lcol);
    } else {
        const EpiCtx c = epi_ctx(p.epi, p.C, p.c_bstride, b);
        MAVG_EPI_DISPATCH(p.epi.kind, (write_tile<KIND, TM, TN>(acc, p.epi, c, p.ldc, p.M, p.N, m0 + wm, n0 + wn, lrow, lcol)))
    }
    if (p.epi.side_sum_src != nullptr && tile == 0 && bz == 0) side_sum(p.epi, &As[0][0][0]);      // (uniform over the workgroup)
}

template <int BM, int BN, int BK, int WM, int WN, int PF, bool AKC, bool BKC>
__global__ __launch_bounds__(64 * WM * WN) void gemm_kernel(GemmKParams p) {
    gemm_body<BM, BN, BK, WM, WN, PF, AKC, BKC>(p, blockIdx.x, blockIdx.z);
}

// ---- 64x64 tile fed by direct global -> LDS loads -------------------------------------------------
//
// The same 2x2 wavefronts of 32x32, but the operand tiles never pass through registers: every wavefront issues
// two global_load_lds_dwordx4 per 16-step k-tile (1 KB of A and 1 KB of B; lane l's 16 bytes land at LDS
// base + 16 l), into a ring of four LDS stages, three tiles ahead.  Addresses are a scalar base that advances
// per tile plus a per-lane 32-bit offset fixed for the whole loop, so the loop holds no vector ALU work
// besides the MFMAs: a wavefront issues in order, and vector instructions queued behind a chain of dependent
// MFMAs (address arithmetic, and the loads that need it) would otherwise wait for that chain.
//
// LDS layouts.  An operand whose contraction index is contiguous in memory keeps its rows: [row][16], the
// 16-byte chunk q of row r stored at chunk position q ^ ((r >> 2) & 3) (a ds_read_b128 serves 16 lanes = 16
// rows per cycle from 64 banks; rows r, r+4, r+8, r+12 start at the same bank, the xor moves their chunks to the
// four different quarters of the 64-byte row: SQ_LDS_BANK_CONFLICT reads zero with it, half of the LDS cycles
// with (r >> 1) & 3); a lane reads one chunk = four contraction steps at once.  An
// operand whose non-contracted index is contiguous is stored [k][64] as it comes and read with ds_read_b32.
// Both feed the same assignment of contraction steps to MFMAs: step c (0..3) of pair p (0..1) multiplies
// k = 8p + c in lanes 0-31 and k = 8p + 4 + c in lanes 32-63.
//
// Schedule of tile t (operands of t already in registers): first four MFMAs; issue the loads of tile t+3;
// wait until the loads of tile t+1 have landed (younger ones stay in flight); barrier; read the operands of
// tile t+1 into the other register set; last four MFMAs, which cover that LDS latency.  The stage that
// receives tile t+3 held tile t-1, whose reads every wavefront finished before the barrier of tile t-1.
//
// The host picks this path only when the loads need no masking: 16-byte aligned operands and strides, row
// counts of m/n-contiguous operands that are multiples of 4 (or padded to one).  Rows or columns past the edge
// of a ragged tile are clamped to the last valid ones (their products are never stored); contraction steps
// past the last whole k-tile (fewer than 16) are multiplied after the loop from operands read element by
// element.
constexpr int kDmaBK = 16;

__device__ __forceinline__ constexpr int chunk_swizzle(int r) { return (r >> 2) & 3; }

// One direct load: 16 bytes per lane from sbase + voff to LDS address lds_byte + 16 * lane.  The LDS base travels
// in M0, which is saved and restored around the instruction.  Written as inline assembly (not the compiler's
// builtin) on purpose: the compiler makes every LDS read wait for all such loads it knows of, which would
// serialise the ring; here the waits are the explicit s_waitcnt vmcnt in the loop.
__device__ __forceinline__ void dma16(uint32_t voff, const float* sbase, uint32_t lds_byte) {
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"(lds_byte), "v"(voff), "s"(sbase)
                 : "memory");
}

// The same load with the LDS base already in M0 and an immediate offset OFF (0 .. 4095 bytes) that the hardware adds
// to BOTH the global address and the LDS address: several loads of a k-tile share one M0 value (their LDS
// destinations OFF apart) and their per-lane offsets are prepared OFF smaller, which takes the M0 traffic (save,
// set, hazard nop, restore: four scalar instructions per load) out of the loop.
__device__ __forceinline__ uint32_t m0_swap(uint32_t v) {
    uint32_t old;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0" : "=&s"(old) : "s"(v) : "memory");
    return old;
}
__device__ __forceinline__ void m0_set(uint32_t v) { asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(v) : "memory"); }
template <int OFF>
__device__ __forceinline__ void dma16_m0(uint32_t voff, const float* sbase) {
    static_assert(OFF >= 0 && OFF < 4096, "immediate offset of a global load");
    asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(sbase), "n"(OFF) : "memory");
}
constexpr int kDmaBias = 4096;      // bytes: per-lane offsets are kept this much larger, the scalar base this much smaller

// Pin a workgroup-uniform 64-bit value to scalar registers (the compiler cannot always prove uniformity, e.g.
// for fields of a kernel-argument array indexed by the workgroup's group number).
__device__ __forceinline__ uint64_t uniform_u64(uint64_t x) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x), hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

template <int TM, int TN, int NST, bool AKC, bool BKC>
__device__ __forceinline__ void gemm_dma_body(const GemmKParams& p, const int tile, const int bz) {
    // workgroup tile BM x BN = (64 TM) x (64 TN): 2x2 wavefronts, each TM x TN accumulators of 32x32
    constexpr int BK = kDmaBK, BM = 64 * TM, BN = 64 * TN;
    static_assert(NST == 3 || NST == 4, "ring of 3 or 4 stages");
    constexpr int TILE_A = BM * BK, TILE_B = BN * BK;          // floats per stage
    constexpr int LOADS = TM + TN;                             // direct loads per wavefront per k-tile
    static_assert(LOADS <= 4, "the vmcnt limits below are written for at most 4 loads per k-tile");
    __shared__ __attribute__((aligned(1024))) float As[NST][TILE_A];
    __shared__ __attribute__((aligned(1024))) float Bs[NST][TILE_B];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane >> 5, lcol = lane & 31;
    const int wm = (wave >> 1) * (32 * TM), wn = (wave & 1) * (32 * TN);
    const int b = bz / p.splits, split = bz - b * p.splits;
    int tm_i, tn_i;
    tile_coords(p, tile, tm_i, tn_i);
    const int m0 = tm_i * BM, n0 = tn_i * BN;
    const int kbeg = split * p.kper;
    const int kend = min(p.K, kbeg + p.kper);
    const int nkt = __builtin_amdgcn_readfirstlane((kend - kbeg) / BK);

    // Direct load number i (0 .. T-1) of this wavefront for an operand of BR = 64 T rows covers the 256 floats
    // [256 (4 i + wave), +256) of the stage.  k-contiguous operand ([row][16]): 16 rows, lane -> row lane/4, chunk
    // position lane%4 (holding chunk position ^ swizzle(row)).  m/n-contiguous operand ([k][BR]): 256/BR k-rows,
    // lane -> k-row lane / (BR/4), columns 4 (lane % (BR/4)).  Returns the lane's byte offset inside the operand.
    auto lane_offset = [&](bool kc, int i, int BR, int r0, int R, int64_t ld) -> uint32_t {
        const int blk = 4 * i + wave;
        if (kc) {
            const int r = blk * 16 + (lane >> 2), q = (lane & 3) ^ chunk_swizzle(r);
            const int row = min(r0 + r, R - 1);
            return (uint32_t)(((int64_t)row * ld + q * 4) * 4);
        }
        const int per = BR / 4;                     // lanes per k-row
        const int k = blk * (256 / BR) + lane / per, col = min(r0 + (lane % per) * 4, R - 4);
        return (uint32_t)(((int64_t)k * ld + col) * 4);
    };
    uint32_t voa[TM], vob[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) voa[i] = lane_offset(AKC, i, BM, m0, AKC ? p.M : p.Mr, p.lda);
#pragma unroll
    for (int i = 0; i < TN; ++i) vob[i] = lane_offset(BKC, i, BN, n0, BKC ? p.N : p.Nr, p.ldb);
    const float* sa = reinterpret_cast<const float*>(uniform_u64(reinterpret_cast<uint64_t>(
        p.A + (int64_t)b * p.a_bstride + (AKC ? (int64_t)kbeg : (int64_t)kbeg * p.lda))));
    const float* sb = reinterpret_cast<const float*>(uniform_u64(reinterpret_cast<uint64_t>(
        p.B + (int64_t)b * p.b_bstride + (BKC ? (int64_t)kbeg : (int64_t)kbeg * p.ldb))));
    const int64_t stepa = (int64_t)uniform_u64((uint64_t)(AKC ? BK : BK * p.lda));
    const int64_t stepb = (int64_t)uniform_u64((uint64_t)(BKC ? BK : BK * p.ldb));
    const uint32_t la = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&As[0][wave * 256]);
    const uint32_t lb = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&Bs[0][wave * 256]);
    auto issue = [&](int t, int stage) {
#pragma unroll
        for (int i = 0; i < TM; ++i) dma16(voa[i], sa + t * stepa, la + stage * (TILE_A * 4) + i * 4096);
#pragma unroll
        for (int i = 0; i < TN; ++i) dma16(vob[i], sb + t * stepb, lb + stage * (TILE_B * 4) + i * 4096);
    };
    // younger k-tiles that may stay in flight while the next one is awaited: NST - 2 tiles of LOADS loads each
    auto wait_next = [&]() {
        constexpr int OUT = LOADS * (NST - 2);
        if constexpr (OUT == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
        else if constexpr (OUT == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
        else if constexpr (OUT == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else if constexpr (OUT == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else { static_assert(OUT == 8, "unexpected number of loads in flight"); asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); }
    };

    // operand reads: float offsets inside a stage, per 32-row block of the wavefront and pair of chunks
    int offa[TM][2], offb[TN][2];
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int ia = wm + i * 32 + lcol;
            offa[i][pr] = AKC ? ia * BK + (((2 * pr + lrow) ^ chunk_swizzle(ia)) * 4) : (8 * pr + 4 * lrow) * BM + ia;
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int ib = wn + j * 32 + lcol;
            offb[j][pr] = BKC ? ib * BK + (((2 * pr + lrow) ^ chunk_swizzle(ib)) * 4) : (8 * pr + 4 * lrow) * BN + ib;
        }
    }
    float fa[2][TM][2][4], fb[2][TN][2][4];
    auto read_frags = [&](auto setc, auto stagec) {
        constexpr int set = decltype(setc)::value, stage = decltype(stagec)::value;
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                if (AKC) {
                    const float4 v = *reinterpret_cast<const float4*>(&As[stage][offa[i][pr]]);
                    fa[set][i][pr][0] = v.x; fa[set][i][pr][1] = v.y; fa[set][i][pr][2] = v.z; fa[set][i][pr][3] = v.w;
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) fa[set][i][pr][c] = As[stage][offa[i][pr] + c * BM];
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (BKC) {
                    const float4 v = *reinterpret_cast<const float4*>(&Bs[stage][offb[j][pr]]);
                    fb[set][j][pr][0] = v.x; fb[set][j][pr][1] = v.y; fb[set][j][pr][2] = v.z; fb[set][j][pr][3] = v.w;
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) fb[set][j][pr][c] = Bs[stage][offb[j][pr] + c * BN];
                }
            }
        }
    };

    floatx16 acc[TM][TN];
    static_for<TM * TN>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        acc[t / TN][t % TN] = floatx16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    });
    // Fused (optionally weighted) row sums of A, by the workgroups of the first tile column: all wavefronts take
    // part, wavefront group rs_grp summing its RS_KPG k-rows of every stage for row rs_row; the groups' partial
    // sums meet in LDS after the loop.  The weights are workgroup-uniform and written by no launch that runs
    // beside this one, so they are read through the constant address space: scalar loads, which cost no vector
    // registers and stay out of the vmcnt bookkeeping of the direct loads.
    constexpr int RS_G = 256 / BM, RS_KPG = BK / RS_G;
    const bool rs_block = !AKC && p.epi.rowsum_dst != nullptr && tn_i == 0;
    const int rs_grp = __builtin_amdgcn_readfirstlane(tid / BM), rs_row = tid % BM;
    float rowsum = 0.f;
    typedef const __attribute__((address_space(4))) float* ConstF;
    const ConstF rw = p.epi.rowsum_w
        ? (ConstF)reinterpret_cast<uintptr_t>(p.epi.rowsum_w + (int64_t)b * p.epi.rowsum_w_bstride + kbeg) : (ConstF)0;

    if (nkt > 0) {
#pragma unroll
        for (int t = 0; t < NST - 1; ++t)
            if (t < nkt) issue(t, t);
        if (nkt >= NST - 1) wait_next();
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
        // MFMAs first .. last - 1 of one half of the k-tile (a half has 4 TM TN of them)
        auto multiply = [&](auto setc, auto prc, const int first, const int last) {
            constexpr int set = decltype(setc)::value, pr = decltype(prc)::value;
            static_for<4 * TM * TN>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                constexpr int c = q / (TM * TN), i = (q / TN) % TM, j = q % TN;
                if (q >= first && q < last)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][i][pr][c], fb[set][j][pr][c], acc[i][j], 0, 0, 0);
            });
        };
        constexpr int NMF = 4 * TM * TN;
        auto step = [&](auto uc, const int t) {
            constexpr int u = decltype(uc)::value % NST;    // stage of tile t
            constexpr int set = decltype(uc)::value & 1;    // register set of tile t
            // The loads of tile t + NST - 1 go out behind the first MFMA of the step and the operand reads for tile
            // t + 1 behind the first half of the MFMAs after the barrier, under cover of the matrix pipe: between the
            // halves only the wait and the barrier remain.  (The loads' stage held tile t - 1, which every wavefront has multiplied.)
            multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 0>{}, 0, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (t + NST - 1 < nkt) issue(t + NST - 1, (u + NST - 1) % NST);
            __builtin_amdgcn_sched_barrier(0);
            multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 0>{}, 1, NMF);
            if (rs_block) {       // the stage is overwritten after the coming barrier: read it before
                const float* a = &As[u][rs_grp * RS_KPG * BM + rs_row];
                if (rw) {
#pragma unroll
                    for (int kk = 0; kk < RS_KPG; ++kk) rowsum += a[kk * BM] * rw[t * BK + rs_grp * RS_KPG + kk];
                } else {
#pragma unroll
                    for (int kk = 0; kk < RS_KPG; ++kk) rowsum += a[kk * BM];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (t + NST - 1 < nkt) wait_next();               // tiles t+2, t+3 may stay in flight
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 1>{}, 0, NMF / 2);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < nkt) read_frags(std::integral_constant<int, set ^ 1>{}, std::integral_constant<int, (u + 1) % NST>{});
            __builtin_amdgcn_sched_barrier(0);
            multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 1>{}, NMF / 2, NMF);
            __builtin_amdgcn_sched_barrier(0);
        };
        constexpr int PERIOD = (NST % 2 == 0) ? NST : 2 * NST;      // stages and register sets repeat together
        for (int t = 0; t < nkt; t += PERIOD) {
            static_for<PERIOD>([&](auto uc) {
                if (t + decltype(uc)::value < nkt) step(uc, t + decltype(uc)::value);
            });
        }
    }

    // Contraction steps past the last whole k-tile of this split (fewer than 16; only the last split has any):
    // operands straight from global memory into registers, element by element, zero past the end.
    const int ktail = kbeg + nkt * BK;
    if (ktail < kend) {
        const float* __restrict__ Ab = p.A + (int64_t)b * p.a_bstride;
        const float* __restrict__ Bb = p.B + (int64_t)b * p.b_bstride;
        static_for<2>([&](auto prc) {
            constexpr int pr = decltype(prc)::value;
            float ta[TM][4], tb[TN][4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int k = ktail + 8 * pr + 4 * lrow + c;
                const bool ok = k < kend;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int m = min(m0 + wm + i * 32 + lcol, p.M - 1);
                    ta[i][c] = ok ? (AKC ? Ab[(int64_t)m * p.lda + k] : Ab[(int64_t)k * p.lda + m]) : 0.f;
                }
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = min(n0 + wn + j * 32 + lcol, p.N - 1);
                    tb[j][c] = ok ? (BKC ? Bb[(int64_t)n * p.ldb + k] : Bb[(int64_t)k * p.ldb + n]) : 0.f;
                }
            }
            if (rs_block && rs_grp == 0) {      // (this thread's row is rs_row, not its MFMA lane's)
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const int k = ktail + 8 * pr + c;
                    if (k < kend && m0 + rs_row < p.M)
                        rowsum += Ab[(int64_t)k * p.lda + m0 + rs_row] * (rw ? rw[k - kbeg] : 1.f);
                }
            }
            static_for<4 * TM * TN>([&](auto qc) {
                constexpr int q = decltype(qc)::value;
                constexpr int c = q / (TM * TN), i = (q / TN) % TM, j = q % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(ta[i][c], tb[j][c], acc[i][j], 0, 0, 0);
            });
        });
    }

    if (rs_block) {       // (workgroup-uniform) the groups' partial sums, added in the order of the groups
        float* red = &As[0][0];
        __syncthreads();
        if (rs_grp > 0) red[(rs_grp - 1) * BM + rs_row] = rowsum;
        __syncthreads();
        if (rs_grp == 0) {
#pragma unroll
            for (int g = 1; g < RS_G; ++g) rowsum += red[(g - 1) * BM + rs_row];
        }
    }
    if (rs_block && rs_grp == 0 && m0 + rs_row < p.M) {
        float* d = p.epi.rowsum_dst + (int64_t)b * p.epi.rowsum_bstride + m0 + rs_row;
        float r = p.epi.rowsum_alpha * rowsum;
        if (p.epi.alpha_dev0) r *= p.epi.alpha_dev0[b];
        if (p.epi.alpha_dev1) r *= p.epi.alpha_dev1[b];
        if (p.epi.rowsum_beta != 0.f) r += p.epi.rowsum_beta * *d;
        *d = r;
        if (p.epi.rowsum_dst2) p.epi.rowsum_dst2[(int64_t)b * p.epi.rowsum2_bstride + m0 + rs_row] += r;
    }
    if (p.splits > 1) {
        Epilogue raw;
        EpiCtx c;
        c.bias = nullptr; c.aux = nullptr; c.C2 = nullptr; c.rowvec = nullptr; c.alpha = 1.f; c.lastcol_dst = nullptr;
        c.C = p.ws + ((int64_t)bz * p.M) * p.N;
        write_tile<EPI_STORE, TM, TN>(acc, raw, c, p.N, p.M, p.N, m0 + wm, n0 + wn, lrow, lcol);
    } else {
        const EpiCtx c = epi_ctx(p.epi, p.C, p.c_bstride, b);
        MAVG_EPI_DISPATCH(p.epi.kind, (write_tile<KIND, TM, TN>(acc, p.epi, c, p.ldc, p.M, p.N, m0 + wm, n0 + wn, lrow, lcol)))
    }
    if (p.epi.side_sum_src != nullptr && tile == 0 && bz == 0) side_sum(p.epi, &As[0][0]);      // (uniform over the workgroup)
}

template <int TM, int TN, int NST, bool AKC, bool BKC>
__global__ __launch_bounds__(256) void gemm_dma_kernel(GemmKParams p) {
    gemm_dma_body<TM, TN, NST, AKC, BKC>(p, blockIdx.x, blockIdx.z);
}

// ---- skinny problems: 32x64 tile, contraction split four ways INSIDE the workgroup ---------------------
//
// A 256-row layer has 128 tiles of 64x64: too few for 256 compute units unless the contraction is split, and a
// split across workgroups costs a pass of partial sums through memory plus a reducer launch per layer.  Here
// the split stays inside the workgroup: 8 wavefronts = 4 k-groups of 2, every k-group multiplies its own
// quarter of the contraction range for the same 32x64 output tile (each wavefront one 32x32 block) out of its
// own ring of LDS stages, with the schedule of gemm_dma_body; at the end the groups' accumulators are added in
// group order through LDS and k-group 0 applies the epilogue.  256 workgroups for a 256x2048 output, two
// wavefronts per SIMD, no partial sums in memory, no reducer.  The price: an A tile serves 2 wavefronts
// instead of 4 (3 direct loads per wavefront and k-tile instead of 2).
constexpr int kKGroups = 4;

// 16-byte chunk q of row r of a k-contiguous tile with BK contraction steps per row sits at chunk position
// q ^ kc_swizzle<BK>(r).  A ds_read_b128 serves 16 lanes = 16 rows per cycle from 64 banks: with 64-byte rows
// (BK = 16) rows r, r+4, r+8, r+12 start at the same bank and need four different chunk positions; with 128-byte
// rows (BK = 32) rows of equal parity do, eight of them.
template <int BK>
__device__ __forceinline__ constexpr int kc_swizzle(int r) { return BK == 16 ? (r >> 2) & 3 : (r >> 1) & 7; }

template <int GW, bool AKC, bool BKC, int KG = kKGroups, int NST = 4, int BK = kDmaBK>
__device__ __forceinline__ void gemm_dma_kg_body(const GemmKParams& p, const int tile, const int bz) {
    // GW wavefronts per k-group: 2 (32x64 tile, one barrier per k-tile) or 1 (32x32 tile: a k-group is a single
    // wavefront with a ring of its own, so the loop needs no barrier at all, only the wavefront's own vmcnt waits).
    // BK contraction steps per k-tile: 16, or 32 (twice the MFMAs per barrier and per round of loads, waits and
    // operand reads: the fixed cost of a k-tile, about 160 cycles against 512 of MFMAs at BK = 16, is paid half as often).
    constexpr int BM = 32, BN = 32 * GW;
    static_assert(GW == 1 || GW == 2, "one or two wavefronts per k-group");
    static_assert(BK == 16 || BK == 32, "16 or 32 contraction steps per k-tile");
    constexpr int TILE_A = BM * BK, TILE_B = BN * BK;
    constexpr int A_LOADS = TILE_A / 256 / GW, B_LOADS = TILE_B / 256 / GW, LOADS = A_LOADS + B_LOADS;   // 1 KB each
    constexpr int NPR = BK / 8;                           // pairs of 16-byte chunks (8 contraction steps) per k-tile
    __shared__ __attribute__((aligned(1024))) float As[KG][NST][TILE_A];
    __shared__ __attribute__((aligned(1024))) float Bs[KG][NST][TILE_B];
    static_assert(NST * TILE_B >= GW * 1024, "a k-group's B ring must hold its accumulators for the final sum");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / GW, gw = wave % GW;
    const int lrow = lane >> 5, lcol = lane & 31;
    const int wn = gw * 32;
    const int b = bz;                                  // the contraction is not split across workgroups here
    int tm_i, tn_i;
    tile_coords(p, tile, tm_i, tn_i);
    const int m0 = tm_i * BM, n0 = tn_i * BN;
    // k-tiles of this k-group: a contiguous share of the K / BK tiles
    const int nkt_all = p.K / BK, base = nkt_all / KG, rem = nkt_all % KG;
    const int nkt = __builtin_amdgcn_readfirstlane(base + (kg < rem ? 1 : 0));
    const int first = kg * base + min(kg, rem);
    const int nloop = base + (rem > 0 ? 1 : 0);        // every wavefront takes part in this many barriers
    const int kbeg = first * BK;

    // Direct loads, in units of 256 floats (1 KB, one load of a wavefront).  k-contiguous operand ([row][BK]): a unit
    // is 256 / BK rows, lane -> row lane / (BK/4), chunk position lane % (BK/4).  m/n-contiguous operand ([k][BR]): a
    // unit is 256 / BR k-rows.  The A stage has TILE_A / 256 units, the B stage TILE_B / 256; a wavefront takes units
    // gw, gw + GW, ...
    auto lane_offset = [&](bool kc, int unit, int BR, int r0, int R, int64_t ld) -> uint32_t {
        if (kc) {
            constexpr int CPR = BK / 4;                   // chunks per row
            const int r = unit * (256 / BK) + lane / CPR, q = (lane % CPR) ^ kc_swizzle<BK>(r);
            const int row = min(r0 + r, R - 1);
            return (uint32_t)(((int64_t)row * ld + q * 4) * 4);
        }
        const int per = BR / 4;
        const int k = unit * (256 / BR) + lane / per, col = min(r0 + (lane % per) * 4, R - 4);
        return (uint32_t)(((int64_t)k * ld + col) * 4);
    };
    // Loads 2j and 2j+1 of an operand share one M0 value: the odd one lands GW KB further on through its immediate
    // offset, and fetches from an address prepared that much smaller.
    constexpr int PAIR_OFF = GW * 1024;
    static_assert(A_LOADS <= 2 && B_LOADS % 2 == 0, "loads are issued in pairs that share an LDS base");
    uint32_t voa[A_LOADS], vob[B_LOADS];
#pragma unroll
    for (int i = 0; i < A_LOADS; ++i)
        voa[i] = lane_offset(AKC, gw + i * GW, BM, m0, AKC ? p.M : p.Mr, p.lda) + kDmaBias - (i & 1) * PAIR_OFF;
#pragma unroll
    for (int i = 0; i < B_LOADS; ++i)
        vob[i] = lane_offset(BKC, gw + i * GW, BN, n0, BKC ? p.N : p.Nr, p.ldb) + kDmaBias - (i & 1) * PAIR_OFF;
    const float* sa = reinterpret_cast<const float*>(uniform_u64(reinterpret_cast<uint64_t>(
        p.A + (int64_t)b * p.a_bstride + (AKC ? (int64_t)kbeg : (int64_t)kbeg * p.lda) - kDmaBias / 4)));
    const float* sb = reinterpret_cast<const float*>(uniform_u64(reinterpret_cast<uint64_t>(
        p.B + (int64_t)b * p.b_bstride + (BKC ? (int64_t)kbeg : (int64_t)kbeg * p.ldb) - kDmaBias / 4)));
    const int64_t stepa = (int64_t)uniform_u64((uint64_t)(AKC ? BK : BK * p.lda));
    const int64_t stepb = (int64_t)uniform_u64((uint64_t)(BKC ? BK : BK * p.ldb));
    const uint32_t la = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&As[kg][0][gw * 256]);
    const uint32_t lb = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&Bs[kg][0][gw * 256]);
    auto issue = [&](int t, int stage) {
        const float* ga = sa + t * stepa;
        const float* gb = sb + t * stepb;
        const uint32_t saved_m0 = m0_swap(la + stage * (TILE_A * 4));
        dma16_m0<0>(voa[0], ga);
        if constexpr (A_LOADS == 2) dma16_m0<PAIR_OFF>(voa[1], ga);
        static_for<B_LOADS / 2>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            m0_set(lb + stage * (TILE_B * 4) + j * 2 * PAIR_OFF);
            dma16_m0<0>(vob[2 * j], gb);
            dma16_m0<PAIR_OFF>(vob[2 * j + 1], gb);
        });
        m0_set(saved_m0);
    };

    // operand reads: MFMA step c (0..3) of pair pr multiplies k = 8 pr + c in lanes 0-31 and k = 8 pr + 4 + c in lanes 32-63
    int offa[NPR], offb[NPR];
#pragma unroll
    for (int pr = 0; pr < NPR; ++pr) {
        const int ia = lcol, ib = wn + lcol;
        offa[pr] = AKC ? ia * BK + (((2 * pr + lrow) ^ kc_swizzle<BK>(ia)) * 4) : (8 * pr + 4 * lrow) * BM + ia;
        offb[pr] = BKC ? ib * BK + (((2 * pr + lrow) ^ kc_swizzle<BK>(ib)) * 4) : (8 * pr + 4 * lrow) * BN + ib;
    }
    float fa[2][NPR][4], fb[2][NPR][4];
    auto read_frags = [&](auto setc, auto stagec) {
        constexpr int set = decltype(setc)::value, stage = decltype(stagec)::value;
#pragma unroll
        for (int pr = 0; pr < NPR; ++pr) {
            if (AKC) {
                const float4 v = *reinterpret_cast<const float4*>(&As[kg][stage][offa[pr]]);
                fa[set][pr][0] = v.x; fa[set][pr][1] = v.y; fa[set][pr][2] = v.z; fa[set][pr][3] = v.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) fa[set][pr][c] = As[kg][stage][offa[pr] + c * BM];
            }
            if (BKC) {
                const float4 v = *reinterpret_cast<const float4*>(&Bs[kg][stage][offb[pr]]);
                fb[set][pr][0] = v.x; fb[set][pr][1] = v.y; fb[set][pr][2] = v.z; fb[set][pr][3] = v.w;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) fb[set][pr][c] = Bs[kg][stage][offb[pr] + c * BN];
            }
        }
    };

    floatx16 acc[1][1];
    acc[0][0] = floatx16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // Contraction steps past the last whole k-tile (fewer than BK) are the last k-group's, straight from global memory,
    // element by element.  Their operands are requested here, ahead of every direct load (so they are the oldest
    // loads in flight and the vmcnt waits of the ring cover them), and multiplied after the loop: the latency of these
    // scattered loads runs beside the loop instead of behind it.
    const bool has_tail = kg == KG - 1 && nkt_all * BK < p.K;      // (uniform over the wavefront)
    float ta[NPR][4], tb[NPR][4];
    if (has_tail) {
        const float* __restrict__ Ab = p.A + (int64_t)b * p.a_bstride;
        const float* __restrict__ Bb = p.B + (int64_t)b * p.b_bstride;
        const int m = min(m0 + lcol, p.M - 1), n = min(n0 + wn + lcol, p.N - 1);
#pragma unroll
        for (int pr = 0; pr < NPR; ++pr)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int k = nkt_all * BK + 8 * pr + 4 * lrow + c;
                const bool ok = k < p.K;
                ta[pr][c] = ok ? (AKC ? Ab[(int64_t)m * p.lda + k] : Ab[(int64_t)k * p.lda + m]) : 0.f;
                tb[pr][c] = ok ? (BKC ? Bb[(int64_t)n * p.ldb + k] : Bb[(int64_t)k * p.ldb + n]) : 0.f;
            }
    }
#pragma unroll
    for (int t = 0; t < NST - 1; ++t)
        if (t < nkt) issue(t, t);
    auto wait_next = [&]() {       // NST - 2 younger k-tiles of LOADS loads each may stay in flight
        constexpr int OUT = LOADS * (NST - 2);
        if constexpr (OUT == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
        else if constexpr (OUT == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else if constexpr (OUT == 9) asm volatile("s_waitcnt vmcnt(9)" ::: "memory");
        else { static_assert(OUT == 12, "unexpected number of loads in flight"); asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); }
    };
    auto group_barrier = [&]() {   // publish the landed tile to the other wavefront of the k-group, if there is one
        if constexpr (GW > 1) __syncthreads();
    };
    if (nkt >= NST - 1) wait_next();
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    group_barrier();
    if (nkt > 0) read_frags(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
    // MFMAs first .. last - 1 of one half of the k-tile (a half has 4 NPR / 2 of them)
    auto multiply = [&](auto setc, auto halfc, const int first, const int last) {
        constexpr int set = decltype(setc)::value, half = decltype(halfc)::value;
#pragma unroll
        for (int q = 0; q < 2 * NPR; ++q) {
            const int pr = half * (NPR / 2) + q / 4, c = q % 4;
            if (q >= first && q < last)
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][pr][c], fb[set][pr][c], acc[0][0], 0, 0, 0);
        }
    };
    auto step = [&](auto uc, const int t) {
        constexpr int u = decltype(uc)::value % NST;      // stage of tile t
        constexpr int set = decltype(uc)::value & 1;      // register set of tile t
        // The loads of tile t + NST - 1 are issued behind the first MFMA of the step, under cover of the matrix pipe:
        // between the two halves only the wait and the barrier remain, during which both wavefronts of the SIMD stand
        // still.  (The loads' stage held tile t - 1, which every wavefront has multiplied.)
        if (t < nkt) multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 0>{}, 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (t + NST - 1 < nkt) issue(t + NST - 1, (u + NST - 1) % NST);
        __builtin_amdgcn_sched_barrier(0);
        if (t < nkt) multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 0>{}, 1, 2 * NPR);
        __builtin_amdgcn_sched_barrier(0);
        if (t + NST - 1 < nkt) wait_next();
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        group_barrier();
        // the second half's operands are in registers already: its first two MFMAs go ahead of the reads for tile t + 1
        if (t < nkt) multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 1>{}, 0, 2);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < nkt) read_frags(std::integral_constant<int, set ^ 1>{}, std::integral_constant<int, (u + 1) % NST>{});
        __builtin_amdgcn_sched_barrier(0);
        if (t < nkt) multiply(std::integral_constant<int, set>{}, std::integral_constant<int, 1>{}, 2, 2 * NPR);
        __builtin_amdgcn_sched_barrier(0);
    };
    constexpr int PERIOD = (NST % 2 == 0) ? NST : 2 * NST;      // stages and register sets repeat together
    for (int t = 0; t < nloop; t += PERIOD) {
        static_for<PERIOD>([&](auto uc) {
            if (t + decltype(uc)::value < nloop) step(uc, t + decltype(uc)::value);
        });
    }

    if (has_tail) {      // the contraction steps past the last whole k-tile, operands requested before the loop
        static_for<NPR>([&](auto prc) {
            constexpr int pr = decltype(prc)::value;
            if (nkt_all * BK + 8 * pr < p.K) {        // (uniform) pairs wholly past the end are skipped
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ta[pr][c], tb[pr][c], acc[0][0], 0, 0, 0);
            }
        });
    }

    // Add the k-groups' accumulators in group order.  Every read of the rings is behind the last barrier of the loop
    // and every load has landed, so each k-group parks its accumulators in its own B ring (1024 floats per wavefront).
    // The sum and the epilogue are shared out: with four k-groups, group g adds up and writes elements 4 g .. 4 g + 3
    // of every lane (rows 8 g .. 8 g + 7 of the 32x32 block), so that all wavefronts work through the tail of the
    // kernel (transcendentals, sampling, the loads and stores of the epilogue) instead of one group in four.
    float* red = &Bs[kg][0][0] + gw * 1024;
    static_for<16>([&](auto vc) { red[decltype(vc)::value * 64 + lane] = acc[0][0][decltype(vc)::value]; });
    __syncthreads();
    static_assert(KG == 4, "the epilogue is shared out in bands of 16 / 4 elements");
    static_for<16>([&](auto vc) {
        constexpr int v = decltype(vc)::value;
        if ((v >> 2) == kg) {       // (uniform over the wavefront)
            float r = (&Bs[0][0][0] + gw * 1024)[v * 64 + lane];
#pragma unroll
            for (int g = 1; g < KG; ++g) r += (&Bs[g][0][0] + gw * 1024)[v * 64 + lane];
            acc[0][0][v] = r;
        }
    });
    const EpiCtx c = epi_ctx(p.epi, p.C, p.c_bstride, b);
    MAVG_EPI_DISPATCH(p.epi.kind, (write_tile<KIND, 1, 1>(acc, p.epi, c, p.ldc, p.M, p.N, m0, n0 + wn, lrow, lcol, kg)))
}

// The 32x64 variant (one workgroup per compute unit) takes k-tiles of 32 steps in a ring of three stages (144 KB of
// LDS); the 32x32 variant keeps 16 steps and four stages so that two workgroups share a compute unit.  A deeper ring
// at 16 steps changed nothing measurable: the loop was not waiting on the depth of its prefetch but paying a fixed
// cost per k-tile.
constexpr int kKgWideBK = 32;
template <int GW, bool AKC, bool BKC>
__global__ __launch_bounds__(64 * kKGroups * GW) void gemm_dma_kg_kernel(GemmKParams p) {
    if constexpr (GW == 2) gemm_dma_kg_body<2, AKC, BKC, kKGroups, 3, kKgWideBK>(p, blockIdx.x, blockIdx.z);
    else gemm_dma_kg_body<1, AKC, BKC, kKGroups, 4, kDmaBK>(p, blockIdx.x, blockIdx.z);
}

// Several independent problems of the same operand layout in one launch (e.g. the weight gradients of all
// layers): workgroup x belongs to the group whose tile range contains it.  Contractions are not split here.
constexpr int kMaxGroups = 8;
struct GemmGroupParams {
    GemmKParams g[kMaxGroups];
    int tile_start[kMaxGroups + 1];
    int ngroups;
};

// The group's parameters where they already are: in the kernel-argument segment (constant memory), read through
// a pointer computed from the group's index, so that fields are fetched by scalar loads when they are needed
// instead of the whole 336-byte record sitting in scalar registers through the main loop (a copy selected with
// compile-time indices did: the loop then ran with spilled scalars, 435 of them in the weight-gradient kernel;
// a run-time index into the by-value argument sends the whole array through private memory).  The table is the
// kernel's first (only) argument, i.e. at offset 0 of the segment.
__device__ __forceinline__ const GemmKParams& group_params(const GemmGroupParams& gp, int& first) {
    int gi = 0;
    first = 0;
    static_for<kMaxGroups - 1>([&](auto ic) {
        constexpr int i = decltype(ic)::value + 1;
        if (i < gp.ngroups && (int)blockIdx.x >= gp.tile_start[i]) { gi = i; first = gp.tile_start[i]; }
    });
    gi = __builtin_amdgcn_readfirstlane(gi);
    typedef const __attribute__((address_space(4))) char* ConstBytes;
    ConstBytes base = (ConstBytes)__builtin_amdgcn_kernarg_segment_ptr();
    typedef const __attribute__((address_space(4))) GemmKParams* ConstParams;
    ConstParams q = (ConstParams)(base + offsetof(GemmGroupParams, g) + (size_t)gi * sizeof(GemmKParams));
    return *(const GemmKParams*)q;
}

template <int BM, int BN, int BK, int WM, int WN, int PF, bool AKC, bool BKC>
__global__ __launch_bounds__(64 * WM * WN) void gemm_grouped_kernel(GemmGroupParams gp) {
    int first;
    const GemmKParams& p = group_params(gp, first);
    gemm_body<BM, BN, BK, WM, WN, PF, AKC, BKC>(p, (int)blockIdx.x - first, blockIdx.z);
}

template <int TM, int TN, int NST, bool AKC, bool BKC>
__global__ __launch_bounds__(256) void gemm_dma_grouped_kernel(GemmGroupParams gp) {
    int first;
    const GemmKParams& p = group_params(gp, first);
    gemm_dma_body<TM, TN, NST, AKC, BKC>(p, (int)blockIdx.x - first, blockIdx.z);
}

// Several thin products C = A B^T (few output columns, long contraction, both operands k-contiguous, plain
// store) in one launch of the in-workgroup-split kernel with 32x32 tiles and four k-groups of one wavefront.
// The table is compact so that 40 problems fit the 4 KB of kernel arguments.
constexpr int kMaxThin = kThinMaxProblems, kThinKGroups = 4;
struct ThinProblem {
    const float* A; const float* B; float* C;
    int64_t lda, ldb, ldc, a_bstride, b_bstride, c_bstride;
    int M, N, K;
};
struct ThinGroupParams {
    ThinProblem g[kMaxThin];
    int tile_start[kMaxThin + 1];
    int ngroups;
};
template <int KG>
__global__ __launch_bounds__(64 * KG) void gemm_thin_grouped_kernel(ThinGroupParams gp) {
    int gi = 0, first = 0;
    static_for<kMaxThin - 1>([&](auto ic) {
        constexpr int i = decltype(ic)::value + 1;
        if (i < gp.ngroups && (int)blockIdx.x >= gp.tile_start[i]) { gi = i; first = gp.tile_start[i]; }
    });
    gi = __builtin_amdgcn_readfirstlane(gi);
    // the problem's record straight from the kernel-argument segment (see group_params)
    typedef const __attribute__((address_space(4))) char* ConstBytes;
    typedef const __attribute__((address_space(4))) ThinProblem* ConstProblem;
    const ThinProblem& t = *(const ThinProblem*)(ConstProblem)((ConstBytes)__builtin_amdgcn_kernarg_segment_ptr() +
                                                              offsetof(ThinGroupParams, g) + (size_t)gi * sizeof(ThinProblem));
    GemmKParams p;
    p.A = t.A; p.lda = t.lda; p.a_bstride = t.a_bstride;
    p.B = t.B; p.ldb = t.ldb; p.b_bstride = t.b_bstride;
    p.C = t.C; p.ldc = t.ldc; p.c_bstride = t.c_bstride;
    p.M = t.M; p.N = t.N; p.K = t.K; p.batch = (int)gridDim.z; p.splits = 1;
    p.kper = (t.K + kDmaBK - 1) / kDmaBK * kDmaBK;
    p.Mr = t.M; p.Nr = t.N;
    p.tiles_m = (t.M + 31) / 32; p.tiles_n = (t.N + 31) / 32;
    p.vecA = 1; p.vecB = 1;
    p.ws = nullptr;
    gemm_dma_kg_body<1, true, true, KG>(p, (int)blockIdx.x - first, blockIdx.z);
}


}  // namespace mavg
