// Per-row reductions over a coefficient block: candidate bounds, rounding slack, constants of the next step
// (paper Section 2, candidate bounds; Section 4.1 for the slack).
#include "device_common.hpp"

namespace gp {

// ------------------------------------------------------------------------------------------------
// Per-row reductions over a block:
//   candidate  sum_j (m_j >= 0 ? m_j*cpos_j : m_j*cneg_j)                   (Section 2, candidate bound)
//   rounding   sum_j |m_j| * max(|xlo_j|,|xhi_j|)                           (slack of the float32 storage)
//   constants of the next step: sum_j max(m_j,0)*kap_j + m_j*bias_c
//   S1 = sum_j |m_j|                                                        (slack of the next accumulation)
// With inference rounding (p.eta) the constants also take sum_j |m_j|*eta_j.  Since |m| = 2*max(m,0) - m this needs no
// sum of its own: eta_j is folded into the two constants of the neuron, kap_j + 2*eta_j and bias_c - eta_j.
// For a block over a plain layer cpos/cneg are the layer's upper/lower interval ends.  A block whose
// coefficients already went through a ReLU substitution holds m = M*slope (M >= 0) or m = M*lam (M < 0)
// over the ReLU's INPUT; the candidate over the ReLU's OUTPUT interval [L,U] that DeepPoly takes before
// the substitution is recovered as M*U = m*(U/slope) =: m*rho and M*L = m*L (L = 0 unless the neuron is
// stably active, where lam = 1), and the intercept term M*del = m*(del/slope) =: m*kap.
// The kernels share this arithmetic (scan_term, scan_finish) and differ in how rows and lanes are laid out; which one
// runs is decided by the row length alone, see launch_scan.
// ------------------------------------------------------------------------------------------------
// The same for the kernels that stage the neurons' constants in LDS, with fewer vector instructions per coefficient
// (every one of them is paid in time here): the staged multiplier pair is (cpos - cneg, cneg), so that the candidate
// term needs no select, m*c(m) = max(m,0)*(cpos - cneg) + m*cneg; and the magnitude of the constant terms, which only
// scales a rounding slack, is not summed per coefficient but bounded per row by S1 * max_j(|bias_j| + kap_j).
template <typename CT>
__device__ __forceinline__ void scan_term_staged(bool has_cand, bool do_consts, CT mf, double dcp, double cn, double X,
                                                 double kp, double be, double& cand, double& absx, double& cst, double& s1) {
    const double m = (double)mf;
    const double am = fabs(m);
    const double mp = fmax(m, 0.0);
    if (has_cand) {
        cand = fma(mp, dcp, fma(m, cn, cand));
        absx = fma(am, X, absx);
    }
    if (do_consts) {
        cst = fma(m, be, fma(mp, kp, cst));
        s1 += am;
    }
}

// The scalars of a row that its bookkeeping reads.  Fetched early (scan_row_fetch) by the kernels that want the
// round trip to overlap with the row's own loads.
struct ScanRow {
    double c, err, best, xmax_self, xmax_a, xmax_b;
    int bi;
    bool frozen;
};
__device__ __forceinline__ ScanRow scan_row_fetch(const ScanParams& p, int r, const RowInfo& ri) {
    ScanRow s;
    if (p.gen) {           // the row starts here: constant = +/- bias, no slack yet
        s.c = (double)(ri.sign * p.g.bias[ri.cs]);
        s.err = 0.0;
    } else {
        s.c = p.c[r];
        s.err = p.err[r];
    }
    s.xmax_self = (p.round_coef > 0.0 && p.xmax_self) ? p.xmax_self[ri.b] : 0.0;
    s.bi = 0; s.best = 0.0; s.frozen = true;
    if (p.update_best && p.cpos) {
        // a task that met the termination criterion keeps the bounds it had at that moment
        s.frozen = p.done && p.done[r >= p.rm.Rc ? r - p.rm.Rc : r];
        s.bi = best_index(p.rm, r);
        s.best = p.gen ? INFINITY : p.best[s.bi];
    }
    s.xmax_a = (p.do_consts && p.xmax_a) ? p.xmax_a[ri.b] : 0.0;
    s.xmax_b = (p.do_consts && p.xmax_b) ? p.xmax_b[ri.b] : 0.0;
    return s;
}
// Per-row bookkeeping after the reductions: rounding slack of the stored coefficients, candidate folded into best,
// constants of the next step added to c, slack of the next accumulation.
__device__ __forceinline__ void scan_finish(const ScanParams& p, int r, int nelem, const ScanRow& s, double t_cand,
                                            double t_absx, double t_cst, double t_cstabs, double t_s1) {
    double c = s.c, err = s.err, best = s.best;
    const bool has_cand = p.update_best && p.cpos;
    double e1 = 0.0;
    if (p.do_consts && p.xmax_a) e1 += p.e1_a * s.xmax_a;
    if (p.do_consts && p.xmax_b) e1 += p.e1_b * s.xmax_b;
    scan_finish_math(nelem, p.round_coef, (p.round_coef > 0.0 && p.xmax_self) ? p.coef_floor * s.xmax_self : 0.0, has_cand,
                     p.do_consts != 0, e1, t_cand, t_absx, t_cst, t_cstabs, t_s1, c, err, best);
    if (has_cand && !s.frozen) p.best[s.bi] = best;
    else if (p.gen && !has_cand) p.best[best_index(p.rm, r)] = INFINITY;
    p.c[r] = c;
    p.err[r] = err;
}

// V consecutive stored coefficients (V = 4: aligned to 4 values)
template <typename CT, int V>
__device__ __forceinline__ void scan_load(const CT* src, CT (&mf)[V]) {
    if constexpr (V == 4 && std::is_same<CT, float>::value) {
        const float4 t = *reinterpret_cast<const float4*>(src);
        mf[0] = t.x; mf[1 % V] = t.y; mf[2 % V] = t.z; mf[3 % V] = t.w;
    } else if constexpr (V == 4) {
        const double2 t0 = reinterpret_cast<const double2*>(src)[0], t1 = reinterpret_cast<const double2*>(src)[1];
        mf[0] = t0.x; mf[1 % V] = t0.y; mf[2 % V] = t1.x; mf[3 % V] = t1.y;
    } else {
        mf[0] = src[0];
    }
}

// The same V coefficients of a row that does not exist yet (p.gen): the start layer's own matrix row, i.e. its filter
// placed in the row's window over the predecessor, times the sign of the row and the predecessor's ReLU substitution
// (Section 2: the neuron's affine expression) - the values and roundings of init_kernel's mode 2 - written to the block
// when a later step reads it.  V = 4: e is a multiple of 4 and the 4 values are channels of one window pixel.
template <int V>
__device__ __forceinline__ void scan_gen(const ScanParams& p, const RowInfo& ri, int r, int nelem, int e, float (&mf)[V]) {
    const GenParams& g = p.g;
    float w[V], gr[V];
#pragma unroll
    for (int k = 0; k < V; ++k) { w[k] = 0.f; gr[k] = 1.f; }
    if (g.dense) {
        const float* ws = g.wt + (size_t)ri.cs * nelem + e;
        const float* gs = g.out_grl ? g.out_grl + (size_t)ri.b * nelem + e : nullptr;
        if constexpr (V == 4) {
            const float4 t = *reinterpret_cast<const float4*>(ws);
            w[0] = t.x; w[1 % V] = t.y; w[2 % V] = t.z; w[3 % V] = t.w;
            if (gs) { const float4 u = *reinterpret_cast<const float4*>(gs); gr[0] = u.x; gr[1 % V] = u.y; gr[2 % V] = u.z; gr[3 % V] = u.w; }
        } else {
            w[0] = ws[0];
            if (gs) gr[0] = gs[0];
        }
    } else {
        const uint32_t pix = fast_div((uint32_t)e, p.div_C);
        const int c = e - (int)pix * g.C;
        const uint32_t a = fast_div(pix, p.div_wx);
        const int A = clampi(g.Sy * ri.ys - g.Py, 0, g.H - g.wy) + (int)a;
        const int B = clampi(g.Sx * ri.xs - g.Px, 0, g.W - g.wx) + (int)(pix - a * (uint32_t)g.wx);
        const int f = A - (ri.ys * g.sh - g.ph), gg = B - (ri.xs * g.sw - g.pw);
        if (f >= 0 && f < g.kh && gg >= 0 && gg < g.kw) {
            const float* ws = g.wt + ((size_t)(f * g.kw + gg) * g.Cs + ri.cs) * g.C + c;
            const float* gs = g.out_grl ? g.out_grl + (size_t)ri.b * ((size_t)g.H * g.W * g.C) + (size_t)(A * g.W + B) * g.C + c : nullptr;
            if constexpr (V == 4) {
                const float4 t = *reinterpret_cast<const float4*>(ws);
                w[0] = t.x; w[1 % V] = t.y; w[2 % V] = t.z; w[3 % V] = t.w;
                if (gs) { const float4 u = *reinterpret_cast<const float4*>(gs); gr[0] = u.x; gr[1 % V] = u.y; gr[2 % V] = u.z; gr[3 % V] = u.w; }
            } else {
                w[0] = ws[0];
                if (gs) gr[0] = gs[0];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        float v = ri.sign * w[k];
        if (g.out_grl && v != 0.f) v = (float)((double)v * (double)relax_factor((double)v, gr[k]));
        mf[k] = v;
    }
    if (p.gen_write) {
        float* dst = const_cast<float*>(p.blk.data) + (size_t)r * nelem + e;
        if constexpr (V == 4) *reinterpret_cast<float4*>(dst) = make_float4(mf[0], mf[1 % V], mf[2 % V], mf[3 % V]);
        else dst[0] = mf[0];
    }
}

constexpr int SCAN_G = 8;     // rows per wave of the 8-lanes-per-row layout

// Short rows: LPR = 8 lanes per row, 8 rows per wave.  Every lane accumulates for its own row (few registers, many
// resident waves) and fetches the constants of its own elements; lanes of different rows that meet the same neuron
// read the same addresses.
// HC / DC: see scan_lds_kernel.
// GEN: the rows are made here (p.gen, see scan_gen).
template <int V, int LPR, typename CT, bool HC, bool DC, bool GEN = false>
__global__ __launch_bounds__(256) void scan_tall_kernel(const ScanParams p) {
    static_assert(!GEN || std::is_same<CT, float>::value, "generated rows are float32 blocks");
    constexpr int RPW = 64 / LPR;                            // rows per wave
    const int tid = threadIdx.x, lane = tid & 63;
    const BlockDesc& B = p.blk;
    const int groups_per_half = (p.rm.Rc + RPW - 1) / RPW;
    const int gidx = blockIdx.x * 4 + (tid >> 6);
    const int nhalves = p.nrows / p.rm.Rc;
    if (gidx >= groups_per_half * nhalves) return;          // whole wave leaves
    const int half = gidx / groups_per_half;
    const int rr0 = (gidx - half * groups_per_half) * RPW;
    const int nvalid = min(RPW, p.rm.Rc - rr0);
    const int k = lane / LPR, sub = lane % LPR;
    const bool valid = k < nvalid;
    const int r = half * p.rm.Rc + rr0 + (valid ? k : 0);
    const int nelem = B.wy * B.wx * B.C;
    const bool full_row = (B.wx == B.W);
    const RowInfo ri = row_info(p.rm, r);
    const int oy = clampi(B.Sy * ri.ys - B.Py, 0, B.H - B.wy), ox = clampi(B.Sx * ri.xs - B.Px, 0, B.W - B.wx);
    const long long bbase = (long long)ri.b * p.batch_stride;
    const CT* src = reinterpret_cast<const CT*>(B.data) + (size_t)r * nelem;
    double cand = 0.0, absx = 0.0, cst = 0.0, cstabs = 0.0, s1 = 0.0;
    if (valid) {
        for (int e = sub * V; e < nelem; e += LPR * V) {
            CT mf[V];
            if constexpr (GEN) scan_gen<V>(p, ri, r, nelem, e, mf);
            else scan_load<CT, V>(src + e, mf);
            int c;
            long long j;
            const int pix = (int)fast_div((uint32_t)e, p.div_C);
            c = e - pix * B.C;
            if (full_row) {
                j = bbase + (long long)oy * B.W * B.C + e;
            } else {
                const int a = (int)fast_div((uint32_t)pix, p.div_wx), bb = pix - a * B.wx;
                j = bbase + ((long long)((oy + a) * B.W + (ox + bb)) * B.C + c);
            }
#pragma unroll
            for (int v = 0; v < V; ++v) {
                double cp = 0.0, cn = 0.0, X = 0.0, kp = 0.0, be = 0.0;
                if constexpr (HC) {
                    cp = p.cpos[j + v];
                    cn = p.cneg[j + v];
                    X = fmax(fabs(p.xlo[j + v]), fabs(p.xhi[j + v]));
                }
                if constexpr (DC) {
                    if (p.kap) kp = p.kap[j + v];
                    if (p.beff) be = p.beff[c + v];
                    if (p.eta) { const double et = p.eta[j + v]; kp += 2.0 * et; be -= et; }
                }
                scan_term(HC, DC, mf[v], cp, cn, X, kp, be, cand, absx, cst, cstabs, s1);
            }
        }
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) {
        cand += __shfl_xor(cand, off, 64);
        absx += __shfl_xor(absx, off, 64);
        cst += __shfl_xor(cst, off, 64);
        cstabs += __shfl_xor(cstabs, off, 64);
        s1 += __shfl_xor(s1, off, 64);
    }
    if (valid && sub == 0) scan_finish(p, r, nelem, scan_row_fetch(p, r, ri), cand, absx, cst, cstabs, s1);
}

// Rows of a few hundred coefficients (dense layers, small windows): 32 rows per work-group, 8 lanes per row.  The
// per-neuron constants of the rows' window are staged ONCE per work-group in LDS (5 doubles per element) instead of
// being fetched by every wave, every lane accumulates for its own row (few registers, many resident waves), and
// lanes of different rows read the same LDS words (broadcast).  Rows of a work-group that do not share box and
// window origin are handled run by run.
constexpr int SCAN_LDS_MAX = 1024;      // longest row whose constants are staged whole (40 KB of LDS)
constexpr int SCAN_TALL_MAX = 64;       // longest row that takes scan_tall_kernel
constexpr int SCAN_PRE_ROWS = 16384;    // launches up to this many rows take the form that requests everything up front
constexpr int SCAN_CHUNK = 512;         // chunk of longer rows (20 KB of LDS: 8 work-groups per CU)
// ROWS per work-group (8 lanes each); the grouping does not touch a row's arithmetic.
// U: row slices (8 lanes x V elements each) whose loads are in flight together.
// CHUNKED: rows longer than SCAN_LDS_MAX are cut into chunks of SCAN_CHUNK coefficients, one work-group per (32 rows,
// chunk); the five sums of a (row, chunk) go to p.partial and scan_combine_kernel adds a row's chunks in order.
// HC / DC: the launch has candidate multipliers (p.cpos) / adds the constants of the next step (p.do_consts).  As
// compile-time constants they leave the loop over a row's coefficients without branches, so that the LDS reads of a
// slice are issued together and their latency passes once per slice instead of once per coefficient.
// PRE: the row fits U slices per lane; they and the row's scalars are requested before the constants are staged, so
// that a launch with few rows (whose time is a chain of memory round trips, not bandwidth) waits for the constants,
// the row and the scalars at once instead of one after the other.  None of this touches a row's arithmetic or its order.
// GEN: the rows are made here (p.gen, see scan_gen).
template <int V, int ROWS, int U, bool CHUNKED, typename CT, bool HC, bool DC, bool PRE = false, bool GEN = false>
__global__ __launch_bounds__(ROWS * 8) void scan_lds_kernel(const ScanParams p) {
    static_assert(!(PRE && CHUNKED), "a chunked row does not fit the lane's registers");
    static_assert(!GEN || std::is_same<CT, float>::value, "generated rows are float32 blocks");
    constexpr int SCAN_LDS_ROWS = ROWS;
    constexpr int NT = ROWS * 8;
    extern __shared__ __attribute__((aligned(16))) double s_const[];     // [5][nelem_pad]
    __shared__ int s_b[SCAN_LDS_ROWS], s_oy[SCAN_LDS_ROWS], s_ox[SCAN_LDS_ROWS];
    // bits of max_j(|bias_j| + kap_j) over the staged constants (non-negative), one slot per parity of the run: a slot
    // is cleared during the following run, two barriers away from both its readers and its next writers
    __shared__ unsigned long long s_qmax[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const BlockDesc& B = p.blk;
    const int nelem = B.wy * B.wx * B.C;
    const int c0 = CHUNKED ? (int)blockIdx.y * SCAN_CHUNK : 0;             // this work-group's element range
    const int c1 = CHUNKED ? min(nelem, c0 + SCAN_CHUNK) : nelem;
    const int npad = CHUNKED ? SCAN_CHUNK : ((nelem + 3) & ~3);
    double* const s_cp = s_const;
    double* const s_cn = s_const + npad;
    double* const s_X = s_const + 2 * npad;
    double* const s_kp = s_const + 3 * npad;
    double* const s_be = s_const + 4 * npad;
    const int gph = (p.rm.Rc + SCAN_LDS_ROWS - 1) / SCAN_LDS_ROWS;      // work-groups per half
    const int half = blockIdx.x / gph;
    const int rr0 = (blockIdx.x - half * gph) * SCAN_LDS_ROWS;
    const int nvalid = min(SCAN_LDS_ROWS, p.rm.Rc - rr0);
    const int kk = wave * 8 + (lane >> 3), sub = lane & 7;
    const bool valid = kk < nvalid;
    const int r = half * p.rm.Rc + rr0 + (valid ? kk : 0);
    const bool full_row = (B.wx == B.W);
    const RowInfo ri = row_info(p.rm, r);
    if (sub == 0 && valid) {
        s_b[kk] = ri.b;
        s_oy[kk] = clampi(B.Sy * ri.ys - B.Py, 0, B.H - B.wy);
        s_ox[kk] = clampi(B.Sx * ri.xs - B.Px, 0, B.W - B.wx);
    }
    if (tid == 0) s_qmax[0] = s_qmax[1] = 0ull;
    const CT* src = reinterpret_cast<const CT*>(B.data) + (size_t)r * nelem;
    auto load_slices = [&](int e0, CT (&mf)[U][V]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * 8 * V;
            if (e < c1) {
                if constexpr (GEN) scan_gen<V>(p, ri, r, nelem, e, mf[u]);
                else scan_load<CT, V>(src + e, mf[u]);
            }
        }
    };
    // (the row's scalars first: the loads behind a dependent one would have to arrive before it could be used)
    CT mf_pre[PRE ? U : 1][PRE ? V : 1];
    ScanRow row_pre;
    if constexpr (PRE) {
        if (valid && sub == 0) row_pre = scan_row_fetch(p, r, ri);
        if (valid) load_slices(c0 + sub * V, mf_pre);
    }
    __syncthreads();
    double cand = 0.0, absx = 0.0, cst = 0.0, cstabs = 0.0, s1 = 0.0;
    auto add_slices = [&](int e0, const CT (&mf)[U][V]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * 8 * V;
            if (e < c1) {
                const int k = e - c0;
                // the slice's constants: V consecutive doubles of each staged array (V = 4: 32-byte aligned)
                double kcp[V], kcn[V], kX[V], kkp[V], kbe[V];
                auto fetch = [&](const double* a, double (&d)[V]) {
                    if constexpr (V == 4) {
                        const double2 t0 = reinterpret_cast<const double2*>(a + k)[0];
                        const double2 t1 = reinterpret_cast<const double2*>(a + k)[1];
                        d[0] = t0.x; d[1 % V] = t0.y; d[2 % V] = t1.x; d[3 % V] = t1.y;
                    } else {
#pragma unroll
                        for (int v = 0; v < V; ++v) d[v] = a[k + v];
                    }
                };
#pragma unroll
                for (int v = 0; v < V; ++v) kcp[v] = kcn[v] = kX[v] = kkp[v] = kbe[v] = 0.0;
                if constexpr (HC) { fetch(s_cp, kcp); fetch(s_cn, kcn); fetch(s_X, kX); }
                if constexpr (DC) { fetch(s_kp, kkp); fetch(s_be, kbe); }
#pragma unroll
                for (int v = 0; v < V; ++v)
                    scan_term_staged(HC, DC, mf[u][v], kcp[v], kcn[v], kX[v], kkp[v], kbe[v], cand, absx, cst, s1);
            }
        }
    };
    int k0 = 0, run = 0;
    while (k0 < nvalid) {                                   // uniform over the work-group
        if (tid == 0) s_qmax[(run & 1) ^ 1] = 0ull;
        const int b0 = s_b[k0], oy0 = s_oy[k0], ox0 = s_ox[k0];
        // end of the run that starts at row k0: every lane tests one row, the first row that differs is found in the
        // ballot (a loop over the rows costs three LDS round trips and a branch per row, 31 times for a dense layer)
        int k1;
        {
            static_assert(SCAN_LDS_ROWS <= 64, "one lane per row");
            const int my = lane < SCAN_LDS_ROWS ? lane : 0;
            const bool same = lane < nvalid && s_b[my] == b0 && s_oy[my] == oy0 && s_ox[my] == ox0;
            const unsigned long long differs = ~__ballot(same);               // lanes >= nvalid differ
            const unsigned long long m = k0 + 1 < 64 ? differs >> (k0 + 1) : 0ull;
            k1 = m ? min(k0 + 1 + (int)__builtin_ctzll(m), nvalid) : nvalid;
        }
        const long long bbase = (long long)b0 * p.batch_stride;
        double qmax = 0.0;
        for (int e = c0 + tid; e < c1; e += NT) {
            int c;
            long long j;
            const int pix = (int)fast_div((uint32_t)e, p.div_C);
            c = e - pix * B.C;
            if (full_row) {
                j = bbase + (long long)oy0 * B.W * B.C + e;
            } else {
                const int a = (int)fast_div((uint32_t)pix, p.div_wx), bb = pix - a * B.wx;
                j = bbase + ((long long)((oy0 + a) * B.W + (ox0 + bb)) * B.C + c);
            }
            double cp = 0.0, cn = 0.0, X = 0.0, kp = 0.0, be = 0.0;
            if constexpr (HC) {
                cp = p.cpos[j];
                cn = p.cneg[j];
                X = fmax(fabs(p.xlo[j]), fabs(p.xhi[j]));
            }
            if constexpr (DC) {
                if (p.kap) kp = p.kap[j];
                if (p.beff) be = p.beff[c];
                if (p.eta) { const double et = p.eta[j]; kp += 2.0 * et; be -= et; }
            }
            const int k = e - c0;
            s_cp[k] = cp - cn; s_cn[k] = cn; s_X[k] = X; s_kp[k] = kp; s_be[k] = be;
            qmax = fmax(qmax, fabs(be) + kp);
        }
        if constexpr (DC) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) qmax = fmax(qmax, __shfl_xor(qmax, off, 64));
            // non-negative doubles order like their bit patterns
            if (lane == 0) atomicMax(&s_qmax[run & 1], (unsigned long long)__double_as_longlong(qmax));
        }
        __syncthreads();
        if (valid && kk >= k0 && kk < k1) {
            const double s1_before = s1;
            if constexpr (PRE) {
                add_slices(c0 + sub * V, mf_pre);
            } else {
                for (int e0 = c0 + sub * V; e0 < c1; e0 += U * 8 * V) {
                    CT mf[U][V];
                    load_slices(e0, mf);
                    add_slices(e0, mf);
                }
            }
            // magnitude of the row's constant terms (scales a rounding slack only): a row lies in exactly one run
            cstabs = (s1 - s1_before) * __longlong_as_double((long long)s_qmax[run & 1]) * (1.0 + 0x1p-50);
        }
        __syncthreads();                                    // the next run overwrites the constants
        k0 = k1;
        ++run;
    }
#pragma unroll
    for (int off = 4; off > 0; off >>= 1) {
        cand += __shfl_xor(cand, off, 64);
        absx += __shfl_xor(absx, off, 64);
        cst += __shfl_xor(cst, off, 64);
        cstabs += __shfl_xor(cstabs, off, 64);
        s1 += __shfl_xor(s1, off, 64);
    }
    if (valid && sub == 0) {
        if constexpr (CHUNKED) {
            double* out = p.partial + ((size_t)r * gridDim.y + blockIdx.y) * 5;
            out[0] = cand; out[1] = absx; out[2] = cst; out[3] = cstabs; out[4] = s1;
        } else if constexpr (PRE) {
            scan_finish(p, r, nelem, row_pre, cand, absx, cst, cstabs, s1);
        } else {
            scan_finish(p, r, nelem, scan_row_fetch(p, r, ri), cand, absx, cst, cstabs, s1);
        }
    }
}

// a row's chunk sums added in chunk order, then the row's bookkeeping
__global__ __launch_bounds__(256) void scan_combine_kernel(const ScanParams p, int nchunks) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= p.nrows) return;
    const double* in = p.partial + (size_t)r * nchunks * 5;
    double t[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int c = 0; c < nchunks; ++c)
#pragma unroll
        for (int q = 0; q < 5; ++q) t[q] += in[c * 5 + q];
    const RowInfo ri = row_info(p.rm, r);
    scan_finish(p, r, p.blk.wy * p.blk.wx * p.blk.C, scan_row_fetch(p, r, ri), t[0], t[1], t[2], t[3], t[4]);
}


// rows whose constants are staged in LDS (up to SCAN_LDS_MAX coefficients whole, longer ones in chunks)
template <typename CT, bool HC, bool DC, bool GEN>
static void launch_scan_lds(const ScanParams& p, hipStream_t s, int nhalves, int nelem, bool vec) {
    if (nelem <= SCAN_LDS_MAX) {
        const size_t lds = (size_t)5 * ((nelem + 3) & ~3) * sizeof(double);
        const int wgs = ((p.rm.Rc + 31) / 32) * nhalves;
        // (which of the forms runs does not touch a row's arithmetic)
        if (vec && nelem <= 512 && p.nrows <= SCAN_PRE_ROWS)
            hipLaunchKernelGGL((scan_lds_kernel<4, 32, 16, false, CT, HC, DC, true, GEN>), dim3(wgs), dim3(256), lds, s, p);
        else if (vec) hipLaunchKernelGGL((scan_lds_kernel<4, 32, 4, false, CT, HC, DC, false, GEN>), dim3(wgs), dim3(256), lds, s, p);
        else hipLaunchKernelGGL((scan_lds_kernel<1, 32, 4, false, CT, HC, DC, false, GEN>), dim3(wgs), dim3(256), lds, s, p);
    } else {
        const int nchunks = (nelem + SCAN_CHUNK - 1) / SCAN_CHUNK;
        const dim3 grid(((p.rm.Rc + 31) / 32) * nhalves, nchunks);
        const size_t lds = (size_t)5 * SCAN_CHUNK * sizeof(double);
        if (vec) hipLaunchKernelGGL((scan_lds_kernel<4, 32, 4, true, CT, HC, DC, false, GEN>), grid, dim3(256), lds, s, p);
        else hipLaunchKernelGGL((scan_lds_kernel<1, 32, 4, true, CT, HC, DC, false, GEN>), grid, dim3(256), lds, s, p);
        hipLaunchKernelGGL(scan_combine_kernel, dim3((p.nrows + 255) / 256), dim3(256), 0, s, p, nchunks);
    }
}

template <typename CT, bool GEN>
static void launch_scan_t(const ScanParams& p, hipStream_t s, int nhalves, int nelem, bool vec) {
    const bool hc = p.cpos != nullptr, dc = p.do_consts != 0;
    // cross-over of the two layouts measured on MI355X (rows of 48: 109 against 126 us for 819 200 rows; 75: 292 against
    // 191 us for 1 310 720 rows; 256: 398 against 135 us for 409 600 rows)
    if (nelem <= SCAN_TALL_MAX || (nelem > SCAN_LDS_MAX && !p.partial)) {
        const int groups = ((p.rm.Rc + SCAN_G - 1) / SCAN_G) * nhalves;
        const dim3 grid((groups + 3) / 4);
        auto go = [&](auto hc_c, auto dc_c) {
            constexpr bool H = decltype(hc_c)::value, D = decltype(dc_c)::value;
            if (vec) hipLaunchKernelGGL((scan_tall_kernel<4, 8, CT, H, D, GEN>), grid, dim3(256), 0, s, p);
            else hipLaunchKernelGGL((scan_tall_kernel<1, 8, CT, H, D, GEN>), grid, dim3(256), 0, s, p);
        };
        if (hc && dc) go(std::true_type{}, std::true_type{});
        else if (hc) go(std::true_type{}, std::false_type{});
        else if (dc) go(std::false_type{}, std::true_type{});
        else go(std::false_type{}, std::false_type{});
    } else {
        if (hc && dc) launch_scan_lds<CT, true, true, GEN>(p, s, nhalves, nelem, vec);
        else if (hc) launch_scan_lds<CT, true, false, GEN>(p, s, nhalves, nelem, vec);
        else if (dc) launch_scan_lds<CT, false, true, GEN>(p, s, nhalves, nelem, vec);
        else launch_scan_lds<CT, false, false, GEN>(p, s, nhalves, nelem, vec);
    }
}

void launch_scan(const ScanParams& p0, hipStream_t s) {
    if (p0.nrows <= 0) return;
    ScanParams p = p0;
    p.div_C = make_fastdiv((uint32_t)p.blk.C);
    p.div_wx = make_fastdiv((uint32_t)p.blk.wx);
    const int nhalves = p.nrows / p.rm.Rc;
    const int nelem = p.blk.wy * p.blk.wx * p.blk.C;
    const bool vec = (p.blk.C & 3) == 0;
    // the layout depends on the row length only, never on how many rows the launch has: a row's sums are formed in
    // the same order whether its box is analysed alone, in a batch, or in a chunk of a batch
    if (p.coef64) launch_scan_t<double, false>(p, s, nhalves, nelem, vec);       // (the host never sets gen with float64 blocks)
    else if (p.gen) launch_scan_t<float, true>(p, s, nhalves, nelem, vec);
    else launch_scan_t<float, false>(p, s, nhalves, nelem, vec);
}

}  // namespace gp
