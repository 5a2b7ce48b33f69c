// HIP kernels of the DeepPoly back-substitution path for gfx950 (MI355X).
//
// Soundness scheme (the explicit-error-term alternative to the paper's interval coefficients,
// Section 4.1): coefficients are stored as ONE float32 value each; products of two float32
// values are exact in float64; sums are accumulated in float64 (MFMA f64); each new coefficient
// is rounded once to float32.  Every rounding is bounded and the bound, multiplied by the largest
// magnitude the neuron can take, is added to a per-row slack `err` that is part of every
// candidate bound.  All rows are upper-bound expressions (lower bounds are taken on -x).
#include "kernels.hpp"

#include <math.h>

namespace gp {

typedef double double4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return min(max(v, lo), hi); }

struct RowInfo {
    int b, ys, xs, cs;
    float sign;
};

__device__ __forceinline__ RowInfo row_info(const RowMap& rm, int r) {
    RowInfo ri;
    int rr = r;
    ri.sign = 1.f;
    if (r >= rm.Rc) {
        rr = r - rm.Rc;
        ri.sign = -1.f;
    }
    long long g = rm.row0 + rr;
    ri.b = (int)(g / rm.n_start);
    int i = (int)(g - (long long)ri.b * rm.n_start);
    int pos = i / rm.Cs;
    ri.cs = i - pos * rm.Cs;
    ri.ys = pos / rm.Ws;
    ri.xs = pos - ri.ys * rm.Ws;
    return ri;
}

// ------------------------------------------------------------------------------------------------
// Crossing an affine layer: per row a transposed convolution from the window in the layer's output
// to the window in its input (Algorithm 1), written as one implicit GEMM over all rows:
//   M = rows * out-window pixels, N = input channels, K = taps * output channels.
// A operand: gathered block values, with a pending ReLU substitution applied on the fly
//            (a * (a>=0 ? gam : lam), exact in float64).
// B operand: filter taps [tap][C_out][C_in].
// float64 MFMA 16x16x4; accumulators D[i][j]: lane l, register r holds i = 4*r + l/16, j = l%16.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN>
__global__ __launch_bounds__(256) void cross_kernel(const CrossParams p) {
    constexpr int BK = 16;
    constexpr int LDA = BM + 4, LDB = BN + 4;
    constexpr int WAVES_N = (BN >= 64) ? 2 : 1;
    constexpr int WAVES_M = 4 / WAVES_N;
    constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
    constexpr int TM = WTM / 16, TN = WTN / 16;
    constexpr int APT = BM / 64;                    // A pixels per thread
    constexpr int BPT = (BK * BN / 4 + 255) / 256;  // B float4 per thread
    static_assert(TM >= 1 && TN >= 1, "tile");

    __shared__ double As[2][BK][LDA];
    __shared__ double Bs[2][BK][LDB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const long long opix = (long long)p.owy * p.owx;
    const long long M = (long long)p.nrows * opix;
    const long long m0 = (long long)blockIdx.x * BM;
    const int n0 = blockIdx.y * BN;
    const int Ck = p.in.C, N = p.Co;
    const int kchunks = (Ck + BK - 1) / BK;
    const int nIt = p.kh * p.kw * kchunks;
    const bool vecA = (Ck & 3) == 0;
    const bool vecB = (N & 3) == 0;
    const bool relax = p.in.gam != nullptr;

    // ---- per-thread pixel bookkeeping for the A gather
    const int q = tid & 3;
    const float* a_base[APT];
    long long a_rbase[APT];
    int a_A[APT], a_B[APT], a_oiy[APT], a_oix[APT];
    bool a_ok[APT];
#pragma unroll
    for (int i = 0; i < APT; ++i) {
        long long m = m0 + (tid >> 2) + 64 * i;
        a_ok[i] = m < M;
        long long mm = a_ok[i] ? m : 0;
        int r = (int)(mm / opix);
        int rem = (int)(mm - (long long)r * opix);
        int a = rem / p.owx, bb = rem - a * p.owx;
        RowInfo ri = row_info(p.rm, r);
        int ooy = clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy);
        int oox = clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx);
        a_A[i] = ooy + a;
        a_B[i] = oox + bb;
        a_oiy[i] = clampi(p.in.Sy * ri.ys - p.in.Py, 0, p.in.H - p.in.wy);
        a_oix[i] = clampi(p.in.Sx * ri.xs - p.in.Px, 0, p.in.W - p.in.wx);
        a_base[i] = p.in.data + (size_t)r * ((size_t)p.in.wy * p.in.wx * Ck);
        a_rbase[i] = (long long)ri.b * ((long long)p.in.H * p.in.W * Ck);
    }

    // global -> register staging holds the raw float32 words only, so that nothing depends on the
    // loads before the MFMA loop of the current tile has been issued; conversion happens at the
    // register -> LDS copy
    float4 a_raw[APT], a_gam[APT], a_lam[APT];
    float4 b_raw[BPT];

    auto load_tiles = [&](int it) {
        const int t = it / kchunks;
        const int d0 = (it - t * kchunks) * BK;
        const int f = t / p.kw, g = t - f * p.kw;
        // A
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            a_raw[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            a_gam[i] = make_float4(1.f, 1.f, 1.f, 1.f);
            a_lam[i] = make_float4(1.f, 1.f, 1.f, 1.f);
            if (!a_ok[i]) continue;
            int yy = a_A[i] + p.ph - f, xx = a_B[i] + p.pw - g;
            if (yy < 0 || xx < 0) continue;
            int y = yy / p.sh, x = xx / p.sw;
            if (y * p.sh != yy || x * p.sw != xx || y >= p.in.H || x >= p.in.W) continue;
            int yi = y - a_oiy[i], xi = x - a_oix[i];
            if (yi < 0 || yi >= p.in.wy || xi < 0 || xi >= p.in.wx) continue;
            const int d = d0 + 4 * q;
            if (d >= Ck) continue;
            const float* src = a_base[i] + ((size_t)(yi * p.in.wx + xi) * Ck + d);
            const long long ridx = a_rbase[i] + ((long long)(y * p.in.W + x) * Ck + d);
            if (vecA) {
                a_raw[i] = *reinterpret_cast<const float4*>(src);
                if (relax) {
                    a_gam[i] = *reinterpret_cast<const float4*>(p.in.gam + ridx);
                    a_lam[i] = *reinterpret_cast<const float4*>(p.in.lam + ridx);
                }
            } else {
                float v[4] = {0.f, 0.f, 0.f, 0.f}, gm[4] = {1.f, 1.f, 1.f, 1.f}, lm[4] = {1.f, 1.f, 1.f, 1.f};
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (d + j < Ck) {
                        v[j] = src[j];
                        if (relax) { gm[j] = p.in.gam[ridx + j]; lm[j] = p.in.lam[ridx + j]; }
                    }
                a_raw[i] = make_float4(v[0], v[1], v[2], v[3]);
                a_gam[i] = make_float4(gm[0], gm[1], gm[2], gm[3]);
                a_lam[i] = make_float4(lm[0], lm[1], lm[2], lm[3]);
            }
        }
        // B
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            b_raw[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            int idx = tid + 256 * i;
            if (idx >= BK * BN / 4) continue;
            int kk = idx / (BN / 4), nq = idx - kk * (BN / 4);
            int d = d0 + kk, n = n0 + 4 * nq;
            if (d >= Ck || n >= N) continue;
            const float* src = p.wt + ((size_t)(t * Ck + d) * N + n);
            if (vecB) {
                b_raw[i] = *reinterpret_cast<const float4*>(src);
            } else {
                float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (n + j < N) v[j] = src[j];
                b_raw[i] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    };

    auto relaxed = [&](float v, float gm, float lm) -> double {
        // coefficient after the pending ReLU substitution; float32 x float32 is exact in float64
        return relax ? (double)v * (double)(v >= 0.f ? gm : lm) : (double)v;
    };

    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < APT; ++i) {
            int pm = (tid >> 2) + 64 * i;
            As[buf][4 * q + 0][pm] = relaxed(a_raw[i].x, a_gam[i].x, a_lam[i].x);
            As[buf][4 * q + 1][pm] = relaxed(a_raw[i].y, a_gam[i].y, a_lam[i].y);
            As[buf][4 * q + 2][pm] = relaxed(a_raw[i].z, a_gam[i].z, a_lam[i].z);
            As[buf][4 * q + 3][pm] = relaxed(a_raw[i].w, a_gam[i].w, a_lam[i].w);
        }
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            int idx = tid + 256 * i;
            if (idx >= BK * BN / 4) continue;
            int kk = idx / (BN / 4), nq = idx - kk * (BN / 4);
            Bs[buf][kk][4 * nq + 0] = (double)b_raw[i].x;
            Bs[buf][kk][4 * nq + 1] = (double)b_raw[i].y;
            Bs[buf][kk][4 * nq + 2] = (double)b_raw[i].z;
            Bs[buf][kk][4 * nq + 3] = (double)b_raw[i].w;
        }
    };

    double4_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = double4_t{0.0, 0.0, 0.0, 0.0};

    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    const int lk = lane >> 4, lm = lane & 15;
    for (int it = 0; it < nIt; ++it) {
        const int buf = it & 1;
        if (it + 1 < nIt) load_tiles(it + 1);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 4) {
            double av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[buf][kk + lk][wm * WTM + i * 16 + lm];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[j] = Bs[buf][kk + lk][wn * WTN + j * 16 + lm];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        if (it + 1 < nIt) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: (+ residual addend) -> one rounding to float32 -> store
    const bool has_add = p.add.data != nullptr;
    const bool add_relax = has_add && p.add.gam != nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const long long m = m0 + wm * WTM + i * 16 + 4 * r4 + lk;
            if (m >= M) continue;
            const float* add_src = nullptr;
            long long add_ridx = 0;
            if (has_add) {
                int r = (int)(m / opix);
                int rem = (int)(m - (long long)r * opix);
                int a = rem / p.owx, bb = rem - a * p.owx;
                RowInfo ri = row_info(p.rm, r);
                int A = clampi(p.oSy * ri.ys - p.oPy, 0, p.Ho - p.owy) + a;
                int B = clampi(p.oSx * ri.xs - p.oPx, 0, p.Wo - p.owx) + bb;
                int ay = A - clampi(p.add.Sy * ri.ys - p.add.Py, 0, p.add.H - p.add.wy);
                int ax = B - clampi(p.add.Sx * ri.xs - p.add.Px, 0, p.add.W - p.add.wx);
                if (ay >= 0 && ay < p.add.wy && ax >= 0 && ax < p.add.wx) {
                    add_src = p.add.data + ((size_t)r * p.add.wy * p.add.wx + (size_t)(ay * p.add.wx + ax)) * N;
                    add_ridx = (long long)ri.b * ((long long)p.Ho * p.Wo * N) + (long long)(A * p.Wo + B) * N;
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * WTN + j * 16 + lm;
                if (n >= N) continue;
                double v = acc[i][j][r4];
                if (add_src) {
                    float av = add_src[n];
                    double ad = (double)av;
                    if (add_relax) ad *= (double)(av >= 0.f ? p.add.gam[add_ridx + n] : p.add.lam[add_ridx + n]);
                    v += ad;
                }
                p.out[(size_t)m * N + n] = (float)v;
            }
        }
    }
}

template <int BM, int BN>
static void launch_cross_t(const CrossParams& p, hipStream_t s) {
    long long M = (long long)p.nrows * p.owy * p.owx;
    dim3 grid((unsigned)((M + BM - 1) / BM), (unsigned)((p.Co + BN - 1) / BN));
    hipLaunchKernelGGL((cross_kernel<BM, BN>), grid, dim3(256), 0, s, p);
}

void launch_cross(const CrossParams& p, hipStream_t s) {
    long long M = (long long)p.nrows * p.owy * p.owx;
    if (M <= 0 || p.Co <= 0) return;
    const int N = p.Co;
    if (N <= 16) { launch_cross_t<128, 16>(p, s); return; }
    if (N <= 32) { launch_cross_t<128, 32>(p, s); return; }
    // enough work-groups to fill 256 compute units?
    long long wg128 = ((M + 127) / 128) * ((N + 127) / 128);
    if (N > 64 && wg128 >= 512) { launch_cross_t<128, 128>(p, s); return; }
    long long wg64 = ((M + 127) / 128) * ((N + 63) / 64);
    if (wg64 >= 512) { launch_cross_t<128, 64>(p, s); return; }
    launch_cross_t<64, 64>(p, s);
}

// ------------------------------------------------------------------------------------------------
// Per-row reductions over a block (one work-group per row):
//   candidate  sum_j (m_j >= 0 ? m_j*U_j : m_j*L_j)                         (Section 2, candidate bound)
//   rounding   sum_j |m_j| * max(|L_j|,|U_j|)                               (slack of the float32 storage)
//   constants of the next step: sum_j max(m_j,0)*del_j + a_j*bias_c, a_j = m_j*(m_j>=0?gam_j:lam_j)
//   S1 = sum_j |a_j|                                                        (slack of the next accumulation)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

__global__ __launch_bounds__(256) void scan_kernel(const ScanParams p) {
    const int r = blockIdx.x;
    const int tid = threadIdx.x;
    const BlockDesc& B = p.blk;
    const RowInfo ri = row_info(p.rm, r);
    const int oy = clampi(B.Sy * ri.ys - B.Py, 0, B.H - B.wy);
    const int ox = clampi(B.Sx * ri.xs - B.Px, 0, B.W - B.wx);
    const int nelem = B.wy * B.wx * B.C;
    const float* src = B.data + (size_t)r * nelem;
    const long long bbase = (long long)ri.b * p.batch_stride;
    double cand = 0, absx = 0, cst = 0, cstabs = 0, s1 = 0;
    for (int e = tid; e < nelem; e += 256) {
        const float mf = src[e];
        if (mf == 0.f) continue;
        const double m = (double)mf;
        int pix = e / B.C, c = e - pix * B.C;
        int a = pix / B.wx, bb = pix - a * B.wx;
        const long long j = bbase + ((long long)((oy + a) * B.W + (ox + bb)) * B.C + c);
        if (p.lo) {
            const double L = p.lo[j], U = p.hi[j];
            cand += (m >= 0.0) ? m * U : m * L;
            absx += fabs(m) * fmax(fabs(L), fabs(U));
        }
        if (p.do_consts) {
            double av = m;
            if (p.gam) {
                av = m * (double)(mf >= 0.f ? p.gam[j] : p.lam[j]);
                if (mf > 0.f && p.del) {
                    double t = m * p.del[j];
                    cst += t;
                    cstabs += t;
                }
            }
            s1 += fabs(av);
            if (p.beff) {
                double t = av * p.beff[c];
                cst += t;
                cstabs += fabs(t);
            }
        }
    }
    __shared__ double red[5][4];
    cand = wave_sum(cand); absx = wave_sum(absx); cst = wave_sum(cst); cstabs = wave_sum(cstabs); s1 = wave_sum(s1);
    if ((tid & 63) == 0) {
        int w = tid >> 6;
        red[0][w] = cand; red[1][w] = absx; red[2][w] = cst; red[3][w] = cstabs; red[4][w] = s1;
    }
    __syncthreads();
    if (tid == 0) {
        cand = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        absx = red[1][0] + red[1][1] + red[1][2] + red[1][3];
        cst = red[2][0] + red[2][1] + red[2][2] + red[2][3];
        cstabs = red[3][0] + red[3][1] + red[3][2] + red[3][3];
        s1 = red[4][0] + red[4][1] + red[4][2] + red[4][3];
        // a sum of n float64 terms in any order is off by at most (n-1)*2^-53*sum|terms|*(1+tiny)
        const double esum = (double)(nelem + 16) * 0x1p-52;
        double c = p.c[r];
        double err = p.err[r];
        // slack of the stored coefficients: |true - stored| <= round_coef*|stored| (+ subnormal floor)
        err += absx * p.round_coef * (1.0 + esum) + (p.round_coef > 0.0 ? 0x1p-140 * (double)nelem : 0.0);
        if (p.update_best && p.lo) {
            double v = c + cand + err;
            v += (fabs(c) + fabs(cand) + err) * 0x1p-50 + absx * esum;
            p.best[r] = fmin(p.best[r], v);
        }
        if (p.do_consts) {
            double cn = c + cst;
            double e1 = 0.0;
            if (p.xmax_a) e1 += p.e1_a * p.xmax_a[ri.b];
            if (p.xmax_b) e1 += p.e1_b * p.xmax_b[ri.b];
            err += cstabs * esum + (fabs(c) + fabs(cst)) * 0x1p-51 + s1 * e1 * (1.0 + esum);
            c = cn;
        }
        err *= (1.0 + 0x1p-48);   // the few float64 operations above
        p.c[r] = c;
        p.err[r] = err;
    }
}

void launch_scan(const ScanParams& p, hipStream_t s) {
    if (p.nrows <= 0) return;
    hipLaunchKernelGGL(scan_kernel, dim3(p.nrows), dim3(256), 0, s, p);
}

// ------------------------------------------------------------------------------------------------
__global__ void init_kernel(const InitParams p) {
    const long long total = (long long)p.nrows * p.nelem;
    for (long long idx = blockIdx.x * (long long)blockDim.x + threadIdx.x; idx < total;
         idx += (long long)gridDim.x * blockDim.x) {
        int r = (int)(idx / p.nelem);
        int e = (int)(idx - (long long)r * p.nelem);
        RowInfo ri = row_info(p.rm, r);
        float v = 0.f;
        if (!p.certify) {
            v = (e == ri.cs) ? ri.sign : 0.f;
        } else {
            // task cs = index among the other classes, block order is H,W,C; classes are numbered C,H,W
            int label = p.labels[ri.b];
            int j = ri.cs + (ri.cs >= label ? 1 : 0);
            int pix = e / p.C, c = e - pix * p.C;
            int chw = c * (p.H * p.W) + pix;
            if (chw == j) v = 1.f;
            else if (chw == label) v = -1.f;
        }
        p.out[idx] = v;
        if (e == 0) {
            p.c[r] = 0.0;
            p.err[r] = 0.0;
            p.best[r] = INFINITY;
        }
    }
}

void launch_init(const InitParams& p, hipStream_t s) {
    long long total = (long long)p.nrows * p.nelem;
    if (total <= 0) return;
    int blocks = (int)fmin((double)((total + 255) / 256), 65536.0);
    hipLaunchKernelGGL(init_kernel, dim3(blocks), dim3(256), 0, s, p);
}

__device__ __forceinline__ void atomic_max_nonneg(double* addr, double v) {
    // non-negative doubles order like their bit patterns
    atomicMax(reinterpret_cast<unsigned long long*>(addr), (unsigned long long)__double_as_longlong(v));
}

__global__ void finalize_kernel(const FinalizeParams p) {
    int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= p.rm.Rc) return;
    long long g = p.rm.row0 + r;
    double u = p.best[r];
    double l = -p.best[p.rm.Rc + r];
    if (!isfinite(u) || !isfinite(l)) *p.flag = 1;
    p.hi[g] = u;
    p.lo[g] = l;
    double x = fmax(fabs(u), fabs(l));
    if (isfinite(x)) atomic_max_nonneg(p.xmax + g / p.rm.n_start, x);
}

void launch_finalize(const FinalizeParams& p, hipStream_t s) {
    if (p.rm.Rc <= 0) return;
    hipLaunchKernelGGL(finalize_kernel, dim3((p.rm.Rc + 255) / 256), dim3(256), 0, s, p);
}

// ReLU layer: intervals [max(l,0), max(u,0)] and the relaxation  lam*x <= relu(x) <= gam*x + del.
// Any gam in [0,1] is sound when del >= max(-gam*l, u - gam*u); gam is the float32 nearest to u/(u-l).
__global__ void relu_kernel(const ReluParams p) {
    long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i >= p.total) return;
    double l = p.plo[i], u = p.phi[i];
    if (!isfinite(l) || !isfinite(u)) *p.flag = 1;
    p.lo[i] = fmax(l, 0.0);
    p.hi[i] = fmax(u, 0.0);
    float g, lam;
    double d = 0.0;
    if (l >= 0.0) { g = 1.f; lam = 1.f; }
    else if (u <= 0.0) { g = 0.f; lam = 0.f; }
    else {
        g = (float)(u / (u - l));
        g = fminf(fmaxf(g, 0.f), 1.f);
        double gd = (double)g;
        double d1 = -gd * l, d2 = u - gd * u;     // each off by a few ulps at most
        d = fmax(d1, d2);
        d = d + (fabs(d) + fabs(u)) * 0x1p-50 + 0x1p-1000;
        lam = (u > -l) ? 1.f : 0.f;
    }
    p.gam[i] = g;
    p.lam[i] = lam;
    p.del[i] = d;
    double x = fmax(u, 0.0);
    if (isfinite(x)) atomic_max_nonneg(p.xmax + i / p.n, x);
}

void launch_relu(const ReluParams& p, hipStream_t s) {
    if (p.total <= 0) return;
    hipLaunchKernelGGL(relu_kernel, dim3((unsigned)((p.total + 255) / 256)), dim3(256), 0, s, p);
}

// Input box [max(c-eps,clip_lo), min(c+eps,clip_hi)], rounded outward in float64, H,W,C order.
__global__ void box_kernel(const BoxParams p) {
    const long long n = (long long)p.C * p.H * p.W;
    long long idx = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (idx >= n * p.batch) return;
    int b = (int)(idx / n);
    int j = (int)(idx - (long long)b * n);   // H,W,C index
    int pix = j / p.C, c = j - pix * p.C;
    double ctr = (double)p.centers[(long long)b * n + (long long)c * (p.H * p.W) + pix];
    double e = (double)p.eps;
    double lo = nextafter(ctr - e, -INFINITY), hi = nextafter(ctr + e, INFINITY);
    lo = fmax(lo, (double)p.clip_lo);
    hi = fmin(hi, (double)p.clip_hi);
    if (lo > hi) {
        if (ctr < (double)p.clip_lo) lo = hi = (double)p.clip_lo;
        else lo = hi = (double)p.clip_hi;
    }
    if (!isfinite(lo) || !isfinite(hi)) *p.flag = 1;
    p.lo[idx] = lo;
    p.hi[idx] = hi;
    double x = fmax(fabs(lo), fabs(hi));
    if (isfinite(x)) atomic_max_nonneg(p.xmax + b, x);
}

void launch_box(const BoxParams& p, hipStream_t s) {
    long long total = (long long)p.C * p.H * p.W * p.batch;
    if (total <= 0) return;
    hipLaunchKernelGGL(box_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
}

__global__ void fill_f64_kernel(double* p, double v, long long n) {
    long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
__global__ void fill_i32_kernel(int* p, int v, long long n) {
    long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
void launch_fill_f64(double* p, double v, long long n, hipStream_t s) {
    if (n > 0) hipLaunchKernelGGL(fill_f64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, v, n);
}
void launch_fill_i32(int* p, int v, long long n, hipStream_t s) {
    if (n > 0) hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, v, n);
}

// margins = -(upper bound of y_j - y_label), rounded down to float32
__global__ void margins_kernel(const double* best, float* margins, long long n, int* flag) {
    long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i >= n) return;
    double m = -best[i];
    if (!isfinite(m)) *flag = 1;
    float f = (float)m;
    if ((double)f > m) f = nextafterf(f, -INFINITY);
    margins[i] = f;
}
void launch_margins(const double* best, float* margins, long long n, int* flag, hipStream_t s) {
    if (n > 0) hipLaunchKernelGGL(margins_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, best, margins, n, flag);
}

__global__ void mfma_check_kernel(const double* A, const double* B, double* D, int K) {
    int l = threadIdx.x;
    double4_t c = {0.0, 0.0, 0.0, 0.0};
    for (int k0 = 0; k0 < K; k0 += 4) {
        double a = A[(l & 15) * K + k0 + (l >> 4)];
        double b = B[(k0 + (l >> 4)) * 16 + (l & 15)];
        c = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    for (int r = 0; r < 4; ++r) D[(4 * r + (l >> 4)) * 16 + (l & 15)] = c[r];
}
void launch_mfma_check(const double* A, const double* B, double* D, int K, hipStream_t s) {
    hipLaunchKernelGGL(mfma_check_kernel, dim3(1), dim3(64), 0, s, A, B, D, K);
}

}  // namespace gp
