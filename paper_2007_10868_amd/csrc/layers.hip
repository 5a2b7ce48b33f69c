// Everything around the two hot kernels: initial expressions, per-layer interval and relaxation kernels, storing of
// bounds, forward interval analysis, the bookkeeping of early termination, instruction self-checks.
#include "device_common.hpp"

namespace gp {

// ------------------------------------------------------------------------------------------------
// Initial expressions (Section 2: the affine layer's own row; Section 4.3: M^{l-1}(x_i) = the filter taps).
//   mode 0: one-hot +/-1 over the start layer itself (sum layers)
//   mode 1: e_j - e_label over the whole last layer (certification rows)
//   mode 2: +/- the row of the start layer's matrix, i.e. its filter placed in the window over the
//           predecessor; constant = +/- bias.  Exact: no rounding.
//   mode 3: minus a caller-given linear form over the whole last layer; constant = minus its offset
// CT: storage type of the coefficients (float, or double: then one element per lane and no rounding at all)
template <typename CT>
__global__ __launch_bounds__(256) void init_kernel(const InitParams p) {
    // block = 4 rows x 64 elements; grid.x over row quadruples, grid.y over element chunks
    constexpr bool F32 = std::is_same<CT, float>::value;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.nrows) return;
    const RowInfo ri = row_info(p.rm, r);
    CT* out = reinterpret_cast<CT*>(p.out) + (size_t)r * p.nelem;
    if (F32 && p.mode == 2 && p.dense && (p.nelem & 3) == 0) {
        // rows of a dense layer's matrix: four coefficients per lane (16-byte loads and stores)
        const float* w = p.wt + (size_t)ri.cs * p.nelem;
        const float* g = p.out_grl ? p.out_grl + (size_t)ri.b * p.nelem : nullptr;
        for (int e = (blockIdx.y * 64 + (threadIdx.x & 63)) * 4; e < p.nelem; e += gridDim.y * 256) {
            const float4 wv = *reinterpret_cast<const float4*>(w + e);
            float v[4] = {ri.sign * wv.x, ri.sign * wv.y, ri.sign * wv.z, ri.sign * wv.w};
            if (g) {
                const float4 gv = *reinterpret_cast<const float4*>(g + e);
                const float gg[4] = {gv.x, gv.y, gv.z, gv.w};
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (v[k] != 0.f) v[k] = (float)((double)v[k] * (double)relax_factor((double)v[k], gg[k]));
            }
            *reinterpret_cast<float4*>(out + e) = make_float4(v[0], v[1], v[2], v[3]);
        }
    } else if (F32 && p.mode == 2 && !p.dense && (p.C & 3) == 0) {
        // the start layer's filter placed in the row's window over the predecessor: four channels of a window pixel per
        // lane (16-byte loads and stores), pixel coordinates without divisions
        const int oy = clampi(p.Sy * ri.ys - p.Py, 0, p.H - p.wy), ox = clampi(p.Sx * ri.xs - p.Px, 0, p.W - p.wx);
        const int fy = ri.ys * p.sh - p.ph, fx = ri.xs * p.sw - p.pw;
        for (int e = (blockIdx.y * 64 + (threadIdx.x & 63)) * 4; e < p.nelem; e += gridDim.y * 256) {
            const uint32_t pix = fast_div((uint32_t)e, p.div_C);
            const int c = e - (int)pix * p.C;
            const uint32_t a = fast_div(pix, p.div_wx);
            const int A = oy + (int)a, B = ox + (int)(pix - a * (uint32_t)p.wx);
            const int f = A - fy, g = B - fx;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (f >= 0 && f < p.kh && g >= 0 && g < p.kw) {
                const float4 wv = *reinterpret_cast<const float4*>(p.wt + ((size_t)(f * p.kw + g) * p.Cs + ri.cs) * p.C + c);
                v[0] = ri.sign * wv.x; v[1] = ri.sign * wv.y; v[2] = ri.sign * wv.z; v[3] = ri.sign * wv.w;
                if (p.out_grl) {
                    const size_t j = (size_t)ri.b * ((size_t)p.H * p.W * p.C) + (size_t)(A * p.W + B) * p.C + c;
                    const float4 gv = *reinterpret_cast<const float4*>(p.out_grl + j);
                    const float gg[4] = {gv.x, gv.y, gv.z, gv.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (v[k] != 0.f) v[k] = (float)((double)v[k] * (double)relax_factor((double)v[k], gg[k]));
                }
            }
            *reinterpret_cast<float4*>(out + e) = make_float4(v[0], v[1], v[2], v[3]);
        }
    } else
    for (int e = blockIdx.y * 64 + (threadIdx.x & 63); e < p.nelem; e += gridDim.y * 64) {
        CT v = 0.f;
        if (p.mode == 0) {
            v = (e == ri.cs) ? ri.sign : 0.f;
        } else if (p.mode == 1) {
            // task cs = index among the other classes, block order is H,W,C; classes are numbered C,H,W
            int label = p.labels[ri.b];
            int j = ri.cs + (ri.cs >= label ? 1 : 0);
            int pix = e / p.C, c = e - pix * p.C;
            int chw = c * (p.H * p.W) + pix;
            if (chw == j) v = 1.f;
            else if (chw == label) v = -1.f;
        } else if (p.mode == 3) {
            // upper bound of minus the form: block order is H,W,C, the form's coefficients are numbered C,H,W
            int pix = e / p.C, c = e - pix * p.C;
            v = -p.forms[(size_t)ri.cs * p.nelem + (size_t)c * (p.H * p.W) + pix];
        } else if (p.dense) {
            v = ri.sign * p.wt[(size_t)ri.cs * p.nelem + e];
            if (p.out_grl && v != 0.f)
                v = (CT)((double)v * (double)relax_factor((double)v, p.out_grl[(size_t)ri.b * p.nelem + e]));
        } else {
            // window over the predecessor (dims H,W,C here), origin from the row's position
            int pix = (int)fast_div((uint32_t)e, p.div_C), c = e - pix * p.C;
            int a = (int)fast_div((uint32_t)pix, p.div_wx), bb = pix - a * p.wx;
            int A = clampi(p.Sy * ri.ys - p.Py, 0, p.H - p.wy) + a;
            int B = clampi(p.Sx * ri.xs - p.Px, 0, p.W - p.wx) + bb;
            int f = A - (ri.ys * p.sh - p.ph), g = B - (ri.xs * p.sw - p.pw);
            if (f >= 0 && f < p.kh && g >= 0 && g < p.kw)
                v = ri.sign * p.wt[((size_t)(f * p.kw + g) * p.Cs + ri.cs) * p.C + c];
            if (p.out_grl && v != 0.f) {
                size_t j = (size_t)ri.b * ((size_t)p.H * p.W * p.C) + (size_t)(A * p.W + B) * p.C + c;
                v = (CT)((double)v * (double)relax_factor((double)v, p.out_grl[j]));
            }
        }
        out[e] = v;
    }
    if (blockIdx.y == 0 && (threadIdx.x & 63) == 0) {
        double c = (p.mode == 2) ? (double)(ri.sign * p.bias[ri.cs]) : (p.mode == 3 && p.offsets) ? -(double)p.offsets[ri.cs] : 0.0;
        // the start neuron's float32 evaluation may exceed its exact expression by eta, in either direction
        if (p.mode == 2 && p.eta)
            c += p.eta[(long long)ri.b * p.rm.n_start + (long long)(ri.ys * p.rm.Ws + ri.xs) * p.rm.Cs + ri.cs] * (1.0 + 0x1p-50);
        p.c[r] = c;
        p.err[r] = 0.0;
        if (!p.seeded) p.best[r] = INFINITY;
    }
}

void launch_init(const InitParams& p0, hipStream_t s) {
    if (p0.nrows <= 0 || p0.nelem <= 0) return;
    InitParams p = p0;
    p.div_C = make_fastdiv((uint32_t)std::max(p.C, 1));
    p.div_wx = make_fastdiv((uint32_t)std::max(p.wx, 1));
    const bool vec4 = !p.coef64 && p.mode == 2 && (p.dense ? (p.nelem & 3) == 0 : (p.C & 3) == 0);
    const int per = vec4 ? p.nelem / 4 : p.nelem;   // items per row
    const int ychunks = (int)fmin((double)((per + 63) / 64), 64.0);
    if (p.coef64) hipLaunchKernelGGL(init_kernel<double>, dim3((p.nrows + 3) / 4, ychunks), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(init_kernel<float>, dim3((p.nrows + 3) / 4, ychunks), dim3(256), 0, s, p);
}

// running maximum of non-negative values, one slot per box; a wave whose lanes all target the same slot
// combines them first (thousands of atomics on one address serialise).  Must be reached by all 64 lanes.
__device__ __forceinline__ void atomic_max_nonneg(double* base, int slot, double v, bool valid) {
    const int first = __builtin_amdgcn_readfirstlane(slot);
    if (__all(valid && slot == first)) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, 64));
        if ((threadIdx.x & 63) == 0)
            atomicMax(reinterpret_cast<unsigned long long*>(base + first), (unsigned long long)__double_as_longlong(v));
    } else if (valid) {
        // non-negative doubles order like their bit patterns
        atomicMax(reinterpret_cast<unsigned long long*>(base + slot), (unsigned long long)__double_as_longlong(v));
    }
}

__global__ void finalize_kernel(const FinalizeParams p) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = r < p.rm.Rc;
    double x = 0.0, xr = 0.0;
    int slot = 0;
    if (valid) {
        const long long g = (long long)p.rm.row0 + r;
        double u = p.best[r];
        double l = -p.best[p.rm.Rc + r];
        if (p.widen > 0.0) {        // the neuron is one rounded float32 addition of the bounded exact sum (monotone)
            u += fabs(u) * p.widen + 0x1p-1000;
            l -= fabs(l) * p.widen + 0x1p-1000;
        }
        if (!isfinite(u) || !isfinite(l)) *p.flag = 1;
        p.hi[g] = u;
        p.lo[g] = l;
        x = fmax(fabs(u), fabs(l));
        if (!isfinite(x)) x = 0.0;
        slot = (int)(g / p.rm.n_start);
        if (p.has_relu) xr = relu_neuron(p.relu, g, l, u);     // (the stored ends, widened if they were)
    }
    atomic_max_nonneg(p.xmax, slot, x, valid);
    if (p.has_relu) atomic_max_nonneg(p.relu.xmax, slot, xr, valid);      // uniform
}

void launch_finalize(const FinalizeParams& p, hipStream_t s) {
    if (p.rm.Rc <= 0) return;
    hipLaunchKernelGGL(finalize_kernel, dim3((p.rm.Rc + 255) / 256), dim3(256), 0, s, p);
}

// ReLU layer: intervals [max(l,0), max(u,0)] and the relaxation  lam*x <= relu(x) <= gam*x + del.
// Any gam in [0,1] is sound when del >= max(-gam*l, u - gam*u); gam is the float32 nearest to u/(u-l).
__global__ void relu_kernel(const ReluParams p) {
    const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    const bool valid = i < p.total;
    double x = 0.0;
    int slot = 0;
    if (valid) {
        x = relu_neuron(p, i, p.plo[i], p.phi[i]);
        slot = (int)(i / p.n);
    }
    atomic_max_nonneg(p.xmax, slot, x, valid);
}

void launch_relu(const ReluParams& p, hipStream_t s) {
    if (p.total <= 0) return;
    hipLaunchKernelGGL(relu_kernel, dim3((unsigned)((p.total + 255) / 256)), dim3(256), 0, s, p);
}

// Input box [max(c-eps,clip_lo), min(c+eps,clip_hi)], rounded outward in float64, H,W,C order.
__global__ void box_kernel(const BoxParams p) {
    const long long n = (long long)p.C * p.H * p.W;
    const long long idx = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    const bool valid = idx < n * p.batch;
    double x = 0.0;
    int b = 0;
    if (valid) {
        b = (int)(idx / n);
        const int j = (int)(idx - (long long)b * n);   // H,W,C index
        const int pix = j / p.C, c = j - pix * p.C;
        const double ctr = (double)p.centers[(long long)b * n + (long long)c * (p.H * p.W) + pix];
        const double e = (double)p.eps;
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
        x = fmax(fabs(lo), fabs(hi));
        if (!isfinite(x)) x = 0.0;
    }
    atomic_max_nonneg(p.xmax, b, x, valid);
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

// ------------------------------------------------------------------------------------------------
// Early termination (Section 3.2: a ReLU input whose interval does not contain 0 strictly gains nothing from
// back-substitution; Section 4.2: forward interval analysis first, only the other rows are back-substituted,
// rows that come to meet the criterion are removed with a prefix sum over the row flags).
// ------------------------------------------------------------------------------------------------
// Interval image of an affine layer: one wave per neuron, float64.  The float32 weight times a float64 bound is
// rounded once (fused multiply-add); a sum of n such terms in any order is off by less than
// (n + 16) * 2^-52 * sum|terms|, which is added outward.
__global__ __launch_bounds__(256) void ival_kernel(const IvalParams p) {
    const int lane = threadIdx.x & 63;
    const long long n = (long long)p.H * p.W * p.C;
    const long long idx = blockIdx.x * 4LL + (threadIdx.x >> 6);
    if (idx >= n * p.batch) return;                         // whole wave leaves
    const int b = (int)(idx / n);
    const int j = (int)(idx - (long long)b * n);
    const int pix = j / p.C, c = j - pix * p.C;
    const int y = pix / p.W, x = pix - y * p.W;
    const long long n_in = (long long)p.Hi * p.Wi * p.Ci;
    const double* plo = p.plo + (long long)b * n_in;
    const double* phi = p.phi + (long long)b * n_in;
    const int taps = p.kh * p.kw;
    double lo = 0.0, hi = 0.0, mag = 0.0;
    for (int t = 0; t < taps; ++t) {
        const int f = t / p.kw, g = t - f * p.kw;
        const int iy = y * p.sh - p.ph + f, ix = x * p.sw - p.pw + g;
        if (iy < 0 || iy >= p.Hi || ix < 0 || ix >= p.Wi) continue;          // uniform per wave
        const float* w = p.wt + ((size_t)t * p.C + c) * p.Ci;
        const double* l = plo + (size_t)(iy * p.Wi + ix) * p.Ci;
        const double* u = phi + (size_t)(iy * p.Wi + ix) * p.Ci;
        for (int ci = lane; ci < p.Ci; ci += 64) {
            const double wv = (double)w[ci], L = l[ci], U = u[ci];
            lo = fma(wv, wv >= 0.0 ? L : U, lo);
            hi = fma(wv, wv >= 0.0 ? U : L, hi);
            mag = fma(fabs(wv), fmax(fabs(L), fabs(U)), mag);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo += __shfl_xor(lo, off, 64);
        hi += __shfl_xor(hi, off, 64);
        mag += __shfl_xor(mag, off, 64);
    }
    if (lane == 0) {
        const double bias = (double)p.bias[c];
        const double terms = (double)taps * p.Ci + 1.0;
        const double slack = (terms + 16.0) * 0x1p-52 * (mag + fabs(bias)) * (1.0 + 0x1p-30);
        double eta = 0.0;
        if (p.eta) {
            // float32 evaluation of sum_j w_j*x_j + bias in any order, fused or not: every term passes through at most
            // `terms` roundings, so |computed - exact| <= gamma(terms)*(sum|w_j||x_j| + |bias|), gamma(k) = k*u/(1-k*u),
            // u = 2^-24, plus half a subnormal step per product that underflows
            const double ku = terms * 0x1p-24;
            const double gamma = ku / (1.0 - ku) * (1.0 + 0x1p-50);
            eta = gamma * (mag * (1.0 + (terms + 16.0) * 0x1p-52) + fabs(bias)) * (1.0 + 0x1p-50) + terms * 0x1p-149;
            if (!isfinite(eta) || ku >= 0.5) *p.flag = 1;
            p.eta[idx] = eta;
        }
        if (p.lo) {
            double l2 = lo + bias - slack - eta, u2 = hi + bias + slack + eta;
            l2 -= fabs(l2) * 0x1p-51 + 0x1p-1000;
            u2 += fabs(u2) * 0x1p-51 + 0x1p-1000;
            if (!isfinite(l2) || !isfinite(u2)) *p.flag = 1;
            p.lo[idx] = l2;
            p.hi[idx] = u2;
        }
    }
}
// the same for an average-pooling layer: one lane per neuron, consecutive lanes are consecutive channels
__global__ __launch_bounds__(256) void pool_ival_kernel(const IvalParams p) {
    const long long n = (long long)p.H * p.W * p.C;
    const long long idx = blockIdx.x * 256LL + threadIdx.x;
    if (idx >= n * p.batch) return;
    const int b = (int)(idx / n);
    const int j = (int)(idx - (long long)b * n);
    const int pix = j / p.C, c = j - pix * p.C;
    const int y = pix / p.W, x = pix - y * p.W;
    const long long n_in = (long long)p.Hi * p.Wi * p.C;
    const double* plo = p.plo + (long long)b * n_in + c;
    const double* phi = p.phi + (long long)b * n_in + c;
    double lo = 0.0, hi = 0.0, mag = 0.0, alo = 0.0, ahi = 0.0;
    for (int f = 0; f < p.kh; ++f) {
        const int iy = y * p.sh - p.ph + f;
        if (iy < 0 || iy >= p.Hi) continue;
        for (int g = 0; g < p.kw; ++g) {
            const int ix = x * p.sw - p.pw + g;
            if (ix < 0 || ix >= p.Wi) continue;
            const double L = plo[(size_t)(iy * p.Wi + ix) * p.C], U = phi[(size_t)(iy * p.Wi + ix) * p.C];
            lo += L; hi += U; alo += fabs(L); ahi += fabs(U); mag += fmax(fabs(L), fabs(U));
        }
    }
    // the scale is 1/(kh*kw) rounded once; the sums carry at most kh*kw - 1 roundings, each relative to the magnitudes
    // summed: a window whose lower ends are all 0 (outputs of ReLUs) keeps the lower end 0 exactly
    const double terms = (double)(p.kh * p.kw) + 1.0;
    const double rel = (terms + 16.0) * 0x1p-52 * p.pool_scale * (1.0 + 0x1p-30);
    mag *= p.pool_scale * (1.0 + 0x1p-50);
    double eta = 0.0;
    if (p.eta) {
        // float32 average: the window summed in any order, then one rounded multiplication by a rounded reciprocal or
        // one rounded division: at most kh*kw + 1 roundings on every term (see ival_kernel)
        const double ku = terms * 0x1p-24;
        const double gamma = ku / (1.0 - ku) * (1.0 + 0x1p-50);
        eta = gamma * mag * (1.0 + (terms + 16.0) * 0x1p-52) * (1.0 + 0x1p-50) + terms * 0x1p-149;
        if (!isfinite(eta) || ku >= 0.5) *p.flag = 1;
        p.eta[idx] = eta;
    }
    if (p.lo) {
        double l2 = lo * p.pool_scale - rel * alo - eta, u2 = hi * p.pool_scale + rel * ahi + eta;
        l2 -= fabs(l2) * 0x1p-51 + (alo > 0.0 ? 0x1p-1000 : 0.0);
        u2 += fabs(u2) * 0x1p-51 + (ahi > 0.0 ? 0x1p-1000 : 0.0);
        if (!isfinite(l2) || !isfinite(u2)) *p.flag = 1;
        p.lo[idx] = l2;
        p.hi[idx] = u2;
    }
}
void launch_ival(const IvalParams& p, hipStream_t s) {
    const long long total = (long long)p.H * p.W * p.C * p.batch;
    if (total <= 0) return;
    if (p.pool_scale != 0.0) {
        hipLaunchKernelGGL(pool_ival_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
        return;
    }
    hipLaunchKernelGGL(ival_kernel, dim3((unsigned)((total + 3) / 4)), dim3(256), 0, s, p);
}

__global__ void add_ival_kernel(const AddIvalParams p) {
    const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i >= p.total) return;
    double l = p.alo[i] + p.blo[i], u = p.ahi[i] + p.bhi[i];
    l -= fabs(l) * (0x1p-52 + p.widen) + 0x1p-1000;
    u += fabs(u) * (0x1p-52 + p.widen) + 0x1p-1000;
    if (!isfinite(l) || !isfinite(u)) *p.flag = 1;
    p.lo[i] = l;
    p.hi[i] = u;
}
void launch_add_ival(const AddIvalParams& p, hipStream_t s) {
    if (p.total <= 0) return;
    hipLaunchKernelGGL(add_ival_kernel, dim3((unsigned)((p.total + 255) / 256)), dim3(256), 0, s, p);
}

__global__ void sum_eta_kernel(const SumEtaParams p) {
    const long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x;
    if (i >= p.total) return;
    double e = 0.0;
    if (p.lo) e = fmax(fabs(p.lo[i]), fabs(p.hi[i])) * p.u;
    if (p.ea) e += p.ea[i];
    if (p.eb) e += p.eb[i];
    p.out[i] = e * (1.0 + 0x1p-50);
}
void launch_sum_eta(const SumEtaParams& p, hipStream_t s) {
    if (p.total <= 0) return;
    hipLaunchKernelGGL(sum_eta_kernel, dim3((unsigned)((p.total + 255) / 256)), dim3(256), 0, s, p);
}

__global__ void seed_kernel(const SeedParams p) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= p.Rc0) return;
    p.best[r] = p.hi[(long long)p.row0 + r];
    p.best[p.Rc0 + r] = -p.lo[(long long)p.row0 + r];
}
void launch_seed(const SeedParams& p, hipStream_t s) {
    if (p.Rc0 <= 0) return;
    hipLaunchKernelGGL(seed_kernel, dim3((p.Rc0 + 255) / 256), dim3(256), 0, s, p);
}

// criterion per task: upper bound <= 0 or lower bound >= 0 (best[Rc0 + .] holds minus the lower bound)
__global__ __launch_bounds__(256) void term_flag_kernel(const TermParams p) {
    __shared__ int s_cnt[4];
    const int rr = blockIdx.x * 256 + threadIdx.x;
    int keep = 0;
    if (rr < p.Ra) {
        const int orig = p.rowid ? p.rowid[rr] : rr;
        const bool was = !p.first && p.done[rr];
        const bool crit = p.may_stop && (p.best[orig] <= 0.0 || p.best[p.Rc0 + orig] <= 0.0);
        const bool now = was || crit;
        p.done[rr] = now ? 1 : 0;
        if (p.term_layer) {
            if (p.first) p.term_layer[(long long)p.row0 + orig] = now ? p.key : 0;
            else if (now && !was) p.term_layer[(long long)p.row0 + orig] = p.key;
        }
        keep = now ? 0 : 1;
    }
    const unsigned long long m = __ballot(keep);
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = __popcll(m);
    __syncthreads();
    if (threadIdx.x == 0) p.wgcount[blockIdx.x] = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
}
// exclusive prefix sum of the per-work-group counts in place (one work-group walks the array), total to *count
__global__ __launch_bounds__(1024) void term_scan_kernel(int* wgcount, int nwg, int* count) {
    __shared__ int s_wave[16];
    __shared__ int s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int base = 0; base < nwg; base += 1024) {
        const int i = base + tid;
        const int v = i < nwg ? wgcount[i] : 0;
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t = __shfl_up(incl, off, 64);
            if (lane >= off) incl += t;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int wave_off = 0;
        for (int w = 0; w < wave; ++w) wave_off += s_wave[w];
        const int carry = s_carry;
        if (i < nwg) wgcount[i] = carry + wave_off + incl - v;
        __syncthreads();
        if (tid == 1023) s_carry = carry + wave_off + incl;
        __syncthreads();
    }
    if (tid == 0) *count = s_carry;
}
void launch_term(const TermParams& p, int* count, hipStream_t s) {
    if (p.Ra <= 0) return;
    const int nwg = (p.Ra + 255) / 256;
    hipLaunchKernelGGL(term_flag_kernel, dim3(nwg), dim3(256), 0, s, p);
    hipLaunchKernelGGL(term_scan_kernel, dim3(1), dim3(1024), 0, s, p.wgcount, nwg, count);
}

__global__ __launch_bounds__(256) void compact_kernel(const CompactParams p) {
    __shared__ int s_cnt[4];
    const int rr = blockIdx.x * 256 + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int keep = (rr < p.Ra && !p.done[rr]) ? 1 : 0;
    const unsigned long long m = __ballot(keep);
    if (lane == 0) s_cnt[wave] = __popcll(m);
    __syncthreads();
    if (!keep) return;
    int pos = p.wgoffset[blockIdx.x] + __popcll(m & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) pos += s_cnt[w];
    const int Ra_new = *p.count;
    p.sel[pos] = rr;
    p.rowid_new[pos] = p.rowid_old ? p.rowid_old[rr] : rr;
    p.done_new[pos] = 0;
    if (p.c_old) {
        for (int h = 0; h < p.nsign; ++h) {
            p.c_new[h * Ra_new + pos] = p.c_old[h * p.Ra + rr];
            p.err_new[h * Ra_new + pos] = p.err_old[h * p.Ra + rr];
        }
    }
}
void launch_compact(const CompactParams& p, hipStream_t s) {
    if (p.Ra <= 0) return;
    hipLaunchKernelGGL(compact_kernel, dim3((p.Ra + 255) / 256), dim3(256), 0, s, p);
}

// block rows of the tasks kept, moved to their new places in another buffer (4 rows per work-group)
__global__ __launch_bounds__(256) void copy_rows_kernel(const CopyRowsParams p) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= p.Ra_new * p.nsign) return;
    const int half = r >= p.Ra_new ? 1 : 0;
    const int i = r - half * p.Ra_new;
    const float* src = p.src + ((size_t)half * p.Ra_old + p.sel[i]) * p.nelem;
    float* dst = p.dst + (size_t)r * p.nelem;
    const int lane = threadIdx.x & 63;
    if ((p.nelem & 3) == 0) {
        const int n4 = p.nelem >> 2;
        for (int e = blockIdx.y * 64 + lane; e < n4; e += gridDim.y * 64)
            reinterpret_cast<float4*>(dst)[e] = reinterpret_cast<const float4*>(src)[e];
    } else {
        for (int e = blockIdx.y * 64 + lane; e < p.nelem; e += gridDim.y * 64) dst[e] = src[e];
    }
}
void launch_copy_rows(const CopyRowsParams& p, hipStream_t s) {
    const long long rows = (long long)p.Ra_new * p.nsign;
    if (rows <= 0 || p.nelem <= 0) return;
    const int per = (p.nelem & 3) == 0 ? p.nelem / 4 : p.nelem;
    const int ychunks = (int)fmin((double)((per + 63) / 64), 32.0);
    hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)((rows + 3) / 4), ychunks), dim3(256), 0, s, p);
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
// the 4-column form used for layers with at most 4 input channels: D[16][4] = A[16][K] * B[K][4]
__global__ void mfma4_check_kernel(const double* A, const double* B, double* D, int K) {
    const int l = threadIdx.x;
    double c = 0.0;
    for (int k0 = 0; k0 < K; k0 += 4) {
        const double a = A[(l & 15) * K + k0 + (l >> 4)];
        const double b = B[(k0 + (l >> 4)) * 4 + (l & 3)];
        c = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, c, 0, 0, 0);
    }
    D[(4 * ((l & 15) >> 2) + (l >> 4)) * 4 + (l & 3)] = c;
}
void launch_mfma4_check(const double* A, const double* B, double* D, int K, hipStream_t s) {
    hipLaunchKernelGGL(mfma4_check_kernel, dim3(1), dim3(64), 0, s, A, B, D, K);
}

}  // namespace gp
