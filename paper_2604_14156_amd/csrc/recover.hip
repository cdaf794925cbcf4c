// Block orthogonal matching pursuit on the GPU (paper Sec. 8 lists greedy pursuit
// restricted to the admissible supports among the per-token solvers; support of
// exactly k units, Sec. 3 / Sec. 7).  One workgroup solves one sketch; the k rounds are sequential.
//
// The rounds run in the Gram domain.  With M = Phi Psi (Sec. 9), G = M^T M and
// c = M^T r, selecting atom a and orthogonalising it against the atoms already
// chosen gives a new orthonormal direction q; the vector d = M^T q obeys
//     d = (G[:,a] - sum_j d_j * d_j[a]) / nrm,    nrm^2 = G[a,a] - sum_j d_j[a]^2,
// the residual loses its component along q:  c <- c - (c[a]/nrm) d,
// and d_j[a_i] (j <= i) is the triangular factor R of the selected atoms (R^T R =
// G_SS), so the refit is a triangular solve.  This is the same greedy sequence and
// the same least-squares refit as the textbook algorithm, at O(N |S|) per round
// instead of O(N m).  After the last round the coefficients are refined once against
// the explicitly formed residual y - M_S alpha, which removes the squared condition
// number the Gram form would otherwise leave in the result.
#include "kernels.hpp"
#include "common.hpp"
#include <math.h>

namespace csk {

struct RecoverLayout {
    int off_corr, off_y, off_r, off_beta, off_alpha, off_gv, off_red, off_selcol, off_order, off_sel;
    int off_gram, off_D;      // -1: lives in global memory
    int total_floats;
};

static RecoverLayout make_layout(const Plan& p, int k, int lds_limit) {
    RecoverLayout L;
    const int N = p.N, m = p.op.m, K = k * p.rb;
    int o = 0;
    L.off_corr = o; o += N;
    L.off_y = o; o += m;
    L.off_r = o; o += m;
    L.off_beta = o; o += K;
    L.off_alpha = o; o += K;
    L.off_gv = o; o += K;
    L.off_red = o; o += 64;
    L.off_selcol = o; o += K;
    L.off_order = o; o += k;
    L.off_sel = o; o += p.G;
    o = (o + 3) & ~3;
    const long limit = lds_limit / 4 - 64;
    L.off_D = -1; L.off_gram = -1;
    if ((long)o + (long)K * N <= limit) { L.off_D = o; o += K * N; }
    o = (o + 3) & ~3;
    if ((long)o + (long)N * N <= limit) { L.off_gram = o; o += N * N; }
    L.total_floats = o;
    return L;
}

size_t recover_spill_floats(const Plan& p, int k, int lds_limit) {
    const RecoverLayout L = make_layout(p, k, lds_limit);
    return L.off_D < 0 ? (size_t)k * p.rb * p.N : 0;
}

struct Top2 { float s1; int i1; float s2; };

__device__ __forceinline__ Top2 top2_merge(const Top2& a, const Top2& b) {
    Top2 o;
    const bool a_wins = (a.s1 > b.s1) || (a.s1 == b.s1 && a.i1 <= b.i1);
    if (a_wins) { o.s1 = a.s1; o.i1 = a.i1; o.s2 = fmaxf(fmaxf(a.s2, b.s2), b.s1); }
    else        { o.s1 = b.s1; o.i1 = b.i1; o.s2 = fmaxf(fmaxf(a.s2, b.s2), a.s1); }
    return o;
}

__global__ void recover_kernel(Plan p, RecoverArgs a, RecoverLayout L) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x, NT = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = NT >> 6;
    const int prob = blockIdx.y * a.B + blockIdx.x;
    if (a.plans) p = a.plans[blockIdx.y];
    const int N = p.N, m = p.op.m, rb = p.rb, G = p.G, k = a.k, K = k * rb;

    float* corr = lds + L.off_corr;
    float* yv = lds + L.off_y;
    float* rv = lds + L.off_r;
    float* beta = lds + L.off_beta;
    float* alpha = lds + L.off_alpha;
    float* gv = lds + L.off_gv;
    float* red = lds + L.off_red;
    int* selcol = reinterpret_cast<int*>(lds + L.off_selcol);
    int* order = reinterpret_cast<int*>(lds + L.off_order);
    int* sel = reinterpret_cast<int*>(lds + L.off_sel);
    // generic pointers: the factor and the Gram matrix live in LDS when they fit
    float* D = L.off_D >= 0 ? lds + L.off_D : a.spill + (size_t)prob * a.spill_stride;
    const float* gram = p.gram;
    if (L.off_gram >= 0) {
        float* gl = lds + L.off_gram;
        for (int i = tid; i < N * N; i += NT) gl[i] = p.gram[i];
        gram = gl;
    }

    const float* y = a.y + (size_t)prob * m;
    int bad_local = 0;
    for (int i = tid; i < m; i += NT) {
        const float v = y[i];
        yv[i] = v;
        if (!isfinite(v)) bad_local = 1;
    }
    for (int g = tid; g < G; g += NT) sel[g] = 0;
    if (tid == 0) { red[60] = 1.0f; red[61] = 0.0f; }       // margin, bad flag
    __syncthreads();
    if (bad_local) red[61] = 1.0f;

    // c = M^T y, one wavefront per atom
    for (int c = wave; c < N; c += nwaves) {
        const float* col = p.Mt + (size_t)c * m;
        float s = 0.f;
        for (int i = lane; i < m; i += 64) s += col[i] * yv[i];
        s = wave_sum(s);
        if (lane == 0) corr[c] = s;
    }
    __syncthreads();

    for (int round = 0; round < k; ++round) {
        // ---- score every unselected unit, keep the best two
        Top2 t; t.s1 = -1.f; t.i1 = 0x7fffffff; t.s2 = -1.f;
        for (int g = tid; g < G; g += NT) {
            if (sel[g]) continue;
            float s = 0.f;
            if (p.weighted) {
                const float* W = p.W + (size_t)g * rb * rb;
                for (int r = 0; r < rb; ++r) {
                    float v = 0.f;
                    for (int c = 0; c <= r; ++c) v += W[r * rb + c] * corr[g * rb + c];
                    s += v * v;
                }
            } else {
                for (int c = 0; c < rb; ++c) { const float v = corr[g * rb + c]; s += v * v; }
            }
            if (!(s >= 0.f)) s = -1.f;                       // NaN never wins
            Top2 u; u.s1 = s; u.i1 = g; u.s2 = -1.f;
            t = top2_merge(t, u);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            Top2 o;
            o.s1 = __shfl_xor(t.s1, off, 64);
            o.i1 = __shfl_xor(t.i1, off, 64);
            o.s2 = __shfl_xor(t.s2, off, 64);
            t = top2_merge(t, o);
        }
        if (lane == 0) { red[wave * 3] = t.s1; red[wave * 3 + 1] = __int_as_float(t.i1); red[wave * 3 + 2] = t.s2; }
        __syncthreads();
        if (tid == 0) {
            Top2 b; b.s1 = red[0]; b.i1 = __float_as_int(red[1]); b.s2 = red[2];
            for (int w = 1; w < nwaves; ++w) {
                Top2 o; o.s1 = red[w * 3]; o.i1 = __float_as_int(red[w * 3 + 1]); o.s2 = red[w * 3 + 2];
                b = top2_merge(b, o);
            }
            int gs = b.i1;
            if (b.s1 < 0.f || gs >= G) {                     // nothing scored: take the first free unit
                gs = 0;
                while (gs < G && sel[gs]) ++gs;
                red[61] = 1.0f;
                red[60] = 0.0f;
            } else {
                const float s2 = fmaxf(b.s2, 0.f);
                const float mg = b.s1 > 0.f ? (b.s1 - s2) / b.s1 : 0.f;
                red[60] = fminf(red[60], mg);
            }
            sel[gs] = 1;
            order[round] = gs;
            red[62] = __int_as_float(gs);
        }
        __syncthreads();
        const int gstar = __float_as_int(red[62]);

        // ---- append the unit's rb atoms to the factor, one at a time
        for (int q = 0; q < rb; ++q) {
            const int col = gstar * rb + q;
            const int J = round * rb + q;
            const float* grow = gram + (size_t)col * N;
            for (int c = tid; c < N; c += NT) {
                float s = 0.f;
                for (int j = 0; j < J; ++j) s += D[(size_t)j * N + c] * D[(size_t)j * N + col];
                D[(size_t)J * N + c] = grow[c] - s;
            }
            __syncthreads();
            const float nrm2 = D[(size_t)J * N + col];
            const float ccol = corr[col];
            const float gdiag = grow[col];
            __syncthreads();
            float inv = 0.f;
            if (nrm2 > 1e-10f * gdiag && nrm2 > 0.f) inv = 1.0f / sqrtf(nrm2);
            const float bt = ccol * inv;
            for (int c = tid; c < N; c += NT) {
                const float dv = D[(size_t)J * N + c] * inv;
                D[(size_t)J * N + c] = dv;
                corr[c] -= bt * dv;
            }
            if (tid == 0) {
                beta[J] = bt;
                selcol[J] = col;
                if (inv == 0.f) red[61] = 1.0f;
            }
            __syncthreads();
        }
    }

    // ---- R alpha = beta, R[j][i] = D[j][selcol[i]] (upper triangular), back substitution
    auto solve_upper = [&](float* rhs, float* out) {
        for (int i = K - 1; i >= 0; --i) {
            const float rii = D[(size_t)i * N + selcol[i]];
            const float v = rii > 0.f ? rhs[i] / rii : 0.f;
            __syncthreads();
            if (tid == 0) out[i] = v;
            for (int j = tid; j < i; j += NT) rhs[j] -= D[(size_t)j * N + selcol[i]] * v;
            __syncthreads();
        }
    };
    // R^T w = rhs (forward substitution), in place
    auto solve_lower_t = [&](float* rhs) {
        for (int i = 0; i < K; ++i) {
            const float rii = D[(size_t)i * N + selcol[i]];
            const float v = rii > 0.f ? rhs[i] / rii : 0.f;
            __syncthreads();
            if (tid == 0) rhs[i] = v;
            for (int l = i + 1 + tid; l < K; l += NT) rhs[l] -= D[(size_t)i * N + selcol[l]] * v;
            __syncthreads();
        }
    };
    solve_upper(beta, alpha);

    // ---- explicit residual r = y - M_S alpha
    for (int i = tid; i < m; i += NT) {
        float s = yv[i];
        for (int j = 0; j < K; ++j) s -= alpha[j] * p.Mt[(size_t)selcol[j] * m + i];
        rv[i] = s;
    }
    __syncthreads();
    // ---- one step of refinement: solve (R^T R) delta = M_S^T r
    for (int j = wave; j < K; j += nwaves) {
        const float* col = p.Mt + (size_t)selcol[j] * m;
        float s = 0.f;
        for (int i = lane; i < m; i += 64) s += col[i] * rv[i];
        s = wave_sum(s);
        if (lane == 0) gv[j] = s;
    }
    __syncthreads();
    solve_lower_t(gv);
    solve_upper(gv, beta);                                   // beta now holds delta
    for (int j = tid; j < K; j += NT) alpha[j] += beta[j];
    float ss = 0.f;
    for (int i = tid; i < m; i += NT) {
        float s = rv[i];
        for (int j = 0; j < K; ++j) s -= beta[j] * p.Mt[(size_t)selcol[j] * m + i];
        ss += s * s;
    }
    ss = wave_sum(ss);
    __syncthreads();
    if (lane == 0) red[wave] = ss;
    __syncthreads();

    // ---- outputs: ascending support, coefficients in that order
    const bool bad = red[61] != 0.f;
    for (int qi = tid; qi < k; qi += NT) {
        const int g = order[qi];
        int rank = 0;
        for (int o = 0; o < k; ++o) rank += order[o] < g;
        a.support[(size_t)prob * k + rank] = g;
        if (a.coef)
            for (int c = 0; c < rb; ++c) a.coef[(size_t)prob * K + rank * rb + c] = alpha[qi * rb + c];
    }
    if (tid == 0) {
        float tot = 0.f;
        for (int w = 0; w < nwaves; ++w) tot += red[w];
        if (a.resid) a.resid[prob] = bad ? __int_as_float(0x7fc00000) : sqrtf(tot);
        if (a.margin) a.margin[prob] = bad ? 0.f : red[60];
    }
}


// ---------------------------------------------------------------------------
// Latency-tuned kernel for one atom per unit (rb == 1) and at most 64 selected
// units.  Thread c owns atom c: its correlation, weight and selection flag live in
// registers and its row of the factor (d_j[c], j = 0..) in LDS.  A round costs one
// workgroup barrier:
//   every wave finds its best and second-best score with lane-crossbar reductions
//   and posts (best, index, second, correlation of the best, reciprocal pivot of the
//   best) to LDS; after the barrier every thread merges the few per-wave candidates
//   itself, so the winner, the margin and the step length are known everywhere
//   without another exchange; the new factor entry needs only the winner's row
//   (broadcast reads) and the thread's own row.  A thread keeps the squared norm of
//   its own factor row in a register, so the pivot of a candidate (its atom's squared
//   norm less that) costs nothing per round.  The single waves that run a round are
//   bound by instruction issue, not by memory: the round is written for few
//   instructions and few separate waits.
// The triangular solves of the refit run inside one wavefront with scalar lane
// broadcasts instead of barriers.
// ---------------------------------------------------------------------------
struct FastLayout {
    int off_y, off_r, off_cand, off_beta, off_alpha, off_gv, off_red, off_selcol, off_Dt, off_gram;
    int KL;               // leading factor entries per atom kept in LDS (the rest in a global spill)
    int KS;               // padded row length of the factor in LDS (floats)
    int rows;             // rows of the factor = atoms rounded up to a wavefront
    int total_floats;
};

constexpr int RF_MAXK = 64;        // selected atoms handled by the single-wavefront solves
constexpr int RF_MAXK_SELECT = 256; // selected atoms of the support-only variant (no solves)
constexpr int RF_THREADS = 512;
constexpr int RP_MIN_PROBLEMS = 256;   // launches with more sketches than this solve two per workgroup

// fit = false (support and margin only): no refit work areas and no padding rows in the factor.
static bool make_fast_layout(const Plan& p, int k, int lds_limit, int nthreads, bool fit, bool have_spill, FastLayout& L) {
    const int N = p.N, m = p.op.m;
    const int kcap = fit ? RF_MAXK : RF_MAXK_SELECT;
    L.rows = fit ? ((N + 63) & ~63) : N;
    int o = 0;
    L.off_y = o; o += (m + 3) & ~3;
    L.off_r = o; if (fit) o += (m + 3) & ~3;
    L.off_cand = o; o += 2 * 16 * 8;
    L.off_beta = o; o += kcap;
    L.off_alpha = o; if (fit) o += RF_MAXK;
    L.off_gv = o; if (fit) o += 16 * RF_MAXK;
    L.off_red = o; o += 16;
    L.off_selcol = o; o += kcap;
    const long limit = lds_limit / 4 - 16;
    auto padded = [](int kl) {
        int ks = (kl + 3) & ~3;
        if (((ks >> 2) & 1) == 0) ks += 4;    // odd number of 16-byte groups per row: conflict-free b128 reads
        return ks;
    };
    // the factor: as many leading entries per atom in LDS as fit; the support-only variant may keep the
    // rest in a global spill (the late rounds then read a few values per atom through L2)
    int KL = k;
    while (KL > 4 && (long)o + (long)L.rows * padded(KL) > limit) KL -= 4;
    if (KL < k && (fit || !have_spill)) return false;
    L.KL = KL;
    L.KS = padded(KL);
    // the factor's storage doubles as the staging area of the initial correlation partial sums
    int dt = L.rows * L.KS;
    const int stage = nthreads * 4;
    if (dt < stage) dt = stage;
    L.off_Dt = o; o += dt;
    L.off_gram = -1;
    if (o > limit) return false;
    if (KL == k && (long)o + (long)N * N <= limit) { L.off_gram = o; o += N * N; }
    L.total_floats = o;
    return true;
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
// maximum of an unsigned key over the wavefront, returned in every lane
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, dpp_u32<CS_DPP_QUAD_SWAP1>(v));
    v = max(v, dpp_u32<CS_DPP_QUAD_SWAP2>(v));
    v = max(v, dpp_u32<CS_DPP_HALF_MIRROR>(v));
    v = max(v, dpp_u32<CS_DPP_ROW_MIRROR>(v));
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
    return max(max(a, b), max(c, d));
}

// WANT_FIT = false is the variant the decode loop runs (support and margin only).  It is held to 128
// registers per lane and, at the 7B FFN shape, below 148 KB of LDS: its eight waves then take half of a
// compute unit's register file and wave slots, and a 16-wave workgroup of a bandwidth-bound kernel from
// another stream (64 registers per lane, a few KB of LDS) fits beside it.
template <bool GRAM_LDS, bool WANT_MARGIN, bool WANT_FIT>
__global__ __launch_bounds__(RF_THREADS) __attribute__((amdgpu_waves_per_eu(WANT_FIT ? 1 : 4, WANT_FIT ? 2 : 4)))
void recover_fast_kernel(Plan p, RecoverArgs a, FastLayout L) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x, NT = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = NT >> 6;
    const int prob = blockIdx.y * a.B + blockIdx.x;
    if (a.plans) p = a.plans[blockIdx.y];
    const int N = p.N, m = p.op.m, k = a.k, KS = L.KS, KL = L.KL;
    const bool active = tid < N;
    const int round_waves = (N + 63) >> 6;     // waves that own atoms

    float* yv = lds + L.off_y;
    float* cand = lds + L.off_cand;            // [2][16][8]
    float* beta = lds + L.off_beta;
    float* alpha = lds + L.off_alpha;
    float* gv = lds + L.off_gv;                // [16][RF_MAXK]
    float* red = lds + L.off_red;
    int* selcol = reinterpret_cast<int*>(lds + L.off_selcol);
    float* Dt = lds + L.off_Dt;                // [rows][KS], row c = factor entries of atom c
    float* gl = lds + L.off_gram;

    // ---- every independent global load is issued before the first wait: the sketch, the
    // score weight, the Gram matrix (to LDS) and the first slice of M for c = M^T y
    const float* y = a.y + (size_t)prob * m;
    const int mrows = (m + NT - 1) / NT;
    float yreg = (tid < m) ? y[tid] : 0.f;
    const float w = (active && p.weighted) ? p.W[tid] : 1.f;
    const float gd = active ? p.gram[(size_t)tid * N + tid] : 1.f;   // squared norm of the thread's atom
    constexpr int GU = WANT_FIT ? 16 : 12;
    const int n4 = (N * N) >> 2;
    float4 greg[GU];
    if (GRAM_LDS) {
        const float4* src = reinterpret_cast<const float4*>(p.gram);
#pragma unroll
        for (int u = 0; u < GU; ++u) {
            const int idx = u * NT + tid;
            greg[u] = idx < n4 ? src[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    // slices of M^T y: a thread takes four adjacent atoms and a contiguous range of rows
    const bool vec4 = (N & 3) == 0;
    const int ncg = vec4 ? (N >> 2) : N;
    const int parts = NT / ncg > 0 ? NT / ncg : 1;
    const int cg = tid % ncg, part = tid / ncg;
    const int rows_per = (m + parts - 1) / parts;
    const int i0 = part * rows_per, i1 = part < parts ? min(m, i0 + rows_per) : i0;
    constexpr int MU = 8;
    float4 mreg[MU];
    if (vec4) {
        const float4* mr = reinterpret_cast<const float4*>(p.Mr) + cg;
#pragma unroll
        for (int u = 0; u < MU; ++u)
            mreg[u] = (i0 + u < i1) ? mr[(size_t)(i0 + u) * ncg] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    int bad = !isfinite(yreg);
    if (tid < m) yv[tid] = yreg;
    for (int i = tid + NT; i < m; i += NT) {          // only when m exceeds the workgroup size
        const float v = y[i];
        yv[i] = v;
        if (!isfinite(v)) bad = 1;
    }
    if (GRAM_LDS) {
        float4* dst = reinterpret_cast<float4*>(gl);
#pragma unroll
        for (int u = 0; u < GU; ++u) {
            const int idx = u * NT + tid;
            if (idx < n4) dst[idx] = greg[u];
        }
        const float4* src = reinterpret_cast<const float4*>(p.gram);
        for (int base = GU * NT; base < n4; base += NT) {     // Gram matrices beyond the first batch
            const int idx = base + tid;
            if (idx < n4) dst[idx] = src[idx];
        }
        for (int i = (n4 << 2) + tid; i < N * N; i += NT) gl[i] = p.gram[i];
    }
    bad = __syncthreads_or(bad);

    float corr = 0.f;
    {
        float* stage = Dt;                              // [parts][N]
        if (vec4) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            const float4* mr = reinterpret_cast<const float4*>(p.Mr) + cg;
            for (int ib = i0; ib < i1; ib += MU) {
                if (ib != i0) {
#pragma unroll
                    for (int u = 0; u < MU; ++u)
                        mreg[u] = (ib + u < i1) ? mr[(size_t)(ib + u) * ncg] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < MU; ++u)
                    if (ib + u < i1) {
                        const float yy = yv[ib + u];
                        acc.x += mreg[u].x * yy; acc.y += mreg[u].y * yy; acc.z += mreg[u].z * yy; acc.w += mreg[u].w * yy;
                    }
            }
            if (part < parts) reinterpret_cast<float4*>(stage)[part * ncg + cg] = acc;
        } else {
            float acc = 0.f;
#pragma unroll 8
            for (int i = i0; i < i1; ++i) acc += p.Mr[(size_t)i * N + cg] * yv[i];
            if (part < parts) stage[part * N + cg] = acc;
        }
        __syncthreads();
        if (active) for (int q = 0; q < parts; ++q) corr += stage[q * N + tid];
        __syncthreads();                                // the staging area becomes the factor
    }
    bool selected = false;
    float margin = 1.f;
    float sq = 0.f;                                     // squared norm of the thread's factor row so far
    float* myrow = Dt + (size_t)(tid < L.rows ? tid : 0) * KS;
    // factor entries beyond the KL kept in LDS: [atom][k - KL] in the global spill of this sketch
    float* spill = (KL < k) ? a.spill + (size_t)prob * a.spill_stride : nullptr;
    float* myspill = spill ? spill + (size_t)(active ? tid : 0) * (k - KL) : nullptr;

    // rows are zero beyond their last written entry, so that a round may read whole groups of four
    for (int i = tid; i < (L.rows * KS) >> 2; i += NT)
        reinterpret_cast<float4*>(Dt)[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int J = 0; J < k; ++J) {
        if (wave < round_waves) {
            // key: 0 for lanes without a candidate, else 1 + the bit pattern of the (non-negative) score
            uint32_t key = 0u;
            if (active && !selected) {
                const float t = w * corr;
                float score = t * t;
                if (!(score >= 0.f)) score = 0.f;        // NaN scores tie at zero
                key = __float_as_uint(score) + 1u;
            }
            const uint32_t m1 = wave_max_u32(key);
            const unsigned long long hit = __ballot(key == m1);
            const int l1 = __ffsll((long long)hit) - 1;
            const float c1 = readlane_f32(corr, l1);
            // the pivot of the wave's candidate: its squared norm less that of its factor row
            const float nrm2 = gd - sq;
            float rs = 0.f;
            if (nrm2 > 1e-10f * gd && nrm2 > 0.f) rs = __builtin_amdgcn_rsqf(nrm2);
            const float i1 = readlane_f32(rs, l1);
            uint32_t m2 = 0u;
            if (WANT_MARGIN) m2 = wave_max_u32(lane == l1 ? 0u : key);
            if (lane == 0) {
                float4 cv;
                cv.x = __uint_as_float(m1); cv.y = __int_as_float(wave * 64 + l1); cv.z = __uint_as_float(m2); cv.w = c1;
                float* cw = cand + ((J & 1) * 16 + wave) * 8;
                *reinterpret_cast<float4*>(cw) = cv;
                cw[4] = i1;
            }
        }
        __syncthreads();
        if (wave < round_waves) {
            const float* cb = cand + (J & 1) * 16 * 8;
            // the waves' candidates are read four at a time and merged by selects: one LDS latency per
            // four waves instead of one (and a branch) per wave
            uint32_t k1 = 0u, k2 = 0u;
            int gstar = 0;
            float ccol = 0.f, inv = 0.f;
            for (int w0 = 0; w0 < round_waves; w0 += 4) {
                float4 cw[4];
                float ci[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (w0 + q < round_waves) {           // uniform: waves without atoms post nothing
                        const float* e = cb + (w0 + q) * 8;
                        cw[q] = *reinterpret_cast<const float4*>(e);
                        ci[q] = e[4];
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (w0 + q >= round_waves) break;
                    const uint32_t o1 = __float_as_uint(cw[q].x);
                    const uint32_t o2 = __float_as_uint(cw[q].z);
                    const bool up = o1 > k1 || w0 + q == 0;   // ties keep the lower wave = lower index
                    k2 = up ? max(max(k2, k1), o2) : max(k2, o1);
                    gstar = up ? __float_as_int(cw[q].y) : gstar;
                    ccol = up ? cw[q].w : ccol;
                    inv = up ? ci[q] : inv;
                    k1 = up ? o1 : k1;
                }
            }
            if (WANT_MARGIN) {
                const float s1 = __uint_as_float(k1 - 1u);
                const float s2 = k2 ? __uint_as_float(k2 - 1u) : 0.f;
                margin = fminf(margin, s1 > 0.f ? (s1 - s2) * __builtin_amdgcn_rcpf(s1) : 0.f);
            }
            if (tid == gstar) selected = true;

            const float* grow = (GRAM_LDS ? gl : p.gram) + (size_t)gstar * N;
            const float gmine = active ? grow[tid] : 0.f;
            const float* prow = Dt + (size_t)gstar * KS;
            float dot = 0.f;
            const int JL = J < KL ? J : KL;            // entries of this round's dot product that sit in LDS
            const int JU = (JL + 3) & ~3;              // in whole groups of four: the rows end in zeros
            // 16 entries per turn, all eight LDS reads issued before the first use: the loop is a chain of
            // LDS latencies otherwise (its trip count is not known at compile time)
            int j = 0;
            for (; j + 16 <= JU; j += 16) {
                float4 u[4], v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u[q] = *reinterpret_cast<const float4*>(myrow + j + 4 * q);
                    v[q] = *reinterpret_cast<const float4*>(prow + j + 4 * q);
                }
                float d2 = 0.f;
#pragma unroll
                for (int q = 0; q < 4; q += 2) {
                    dot += u[q].x * v[q].x + u[q].y * v[q].y + u[q].z * v[q].z + u[q].w * v[q].w;
                    d2 += u[q + 1].x * v[q + 1].x + u[q + 1].y * v[q + 1].y + u[q + 1].z * v[q + 1].z + u[q + 1].w * v[q + 1].w;
                }
                dot += d2;
            }
            if (j < JU) {                               // one to three groups left, read together as well
                const float4 u0 = *reinterpret_cast<const float4*>(myrow + j);
                const float4 v0 = *reinterpret_cast<const float4*>(prow + j);
                if (j + 4 < JU) {
                    const float4 u1 = *reinterpret_cast<const float4*>(myrow + j + 4);
                    const float4 v1 = *reinterpret_cast<const float4*>(prow + j + 4);
                    if (j + 8 < JU) {
                        const float4 u2 = *reinterpret_cast<const float4*>(myrow + j + 8);
                        const float4 v2 = *reinterpret_cast<const float4*>(prow + j + 8);
                        dot += u2.x * v2.x + u2.y * v2.y + u2.z * v2.z + u2.w * v2.w;
                    }
                    dot += u1.x * v1.x + u1.y * v1.y + u1.z * v1.z + u1.w * v1.w;
                }
                dot += u0.x * v0.x + u0.y * v0.y + u0.z * v0.z + u0.w * v0.w;
            }
            if (!GRAM_LDS && J > KL) {                  // a Gram matrix in LDS means the whole factor is too
                const float* pspill = spill + (size_t)gstar * (k - KL);
                for (int j = 0; j < J - KL; ++j) dot += myspill[j] * pspill[j];
            }
            if (inv == 0.f) bad = 1;
            const float dv = (gmine - dot) * inv;
            const float bt = ccol * inv;
            corr -= bt * dv;
            sq += dv * dv;
            if (active) {                                 // lanes without an atom have no row of their own
                if (GRAM_LDS || J < KL) myrow[J] = dv; else myspill[J - KL] = dv;
            }
            if (WANT_FIT && tid == 0) { beta[J] = bt; selcol[J] = gstar; }
        }
    }
    bad = __syncthreads_or(bad);

    if (WANT_FIT) {
        // R[j][i] = Dt[selcol[i]][j] (j <= i).  One wavefront solves the triangular systems: lane l
        // holds component l, row l of R (upper solve) and column l of R (transposed solve) in
        // registers, and the pivots travel by scalar lane reads.
        float rrow[RF_MAXK], rcol[RF_MAXK], rinv = 0.f;
        if (wave == 0) {
            const bool lk = lane < k;
            const float* own = Dt + (size_t)selcol[lk ? lane : 0] * KS;
#pragma unroll
            for (int i = 0; i < RF_MAXK; i += 4) {
                const float4 v = (i < k) ? *reinterpret_cast<const float4*>(own + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                rcol[i] = (lk && i < lane) ? v.x : 0.f;
                rcol[i + 1] = (lk && i + 1 < lane) ? v.y : 0.f;
                rcol[i + 2] = (lk && i + 2 < lane) ? v.z : 0.f;
                rcol[i + 3] = (lk && i + 3 < lane) ? v.w : 0.f;
            }
#pragma unroll
            for (int i = 0; i < RF_MAXK; ++i)
                rrow[i] = (i < k && lk && i > lane) ? Dt[(size_t)selcol[i] * KS + lane] : 0.f;
            const float rd = lk ? own[lane] : 0.f;
            rinv = rd > 0.f ? 1.0f / rd : 0.f;
        }
        auto solve_upper = [&](float rhs) -> float {      // R x = rhs, back substitution
            float x = 0.f;
#pragma unroll
            for (int i = RF_MAXK - 1; i >= 0; --i) {
                if (i < k) {
                    const float xi = readlane_f32(rhs, i) * readlane_f32(rinv, i);
                    x = lane == i ? xi : x;
                    rhs -= rrow[i] * xi;
                }
            }
            return x;
        };
        auto solve_lower_t = [&](float rhs) -> float {    // R^T x = rhs, forward substitution
            float x = 0.f;
#pragma unroll
            for (int i = 0; i < RF_MAXK; ++i) {
                if (i < k) {
                    const float xi = readlane_f32(rhs, i) * readlane_f32(rinv, i);
                    x = lane == i ? xi : x;
                    rhs -= rcol[i] * xi;
                }
            }
            return x;
        };
        if (wave == 0) {
            const float x = solve_upper(lane < k ? beta[lane] : 0.f);
            if (lane < k) alpha[lane] = x;
        }
        __syncthreads();
        // explicit residual; thread i keeps its row of M_S in registers for the second pass
        const bool one_row = mrows == 1;
        float mv[RF_MAXK];
        float racc = 0.f;
        float* rv = lds + L.off_r;
        if (one_row) {
            if (tid < m) {
#pragma unroll
                for (int j = 0; j < RF_MAXK; ++j) mv[j] = j < k ? p.Mr[(size_t)tid * N + selcol[j]] : 0.f;
                racc = yv[tid];
#pragma unroll
                for (int j = 0; j < RF_MAXK; ++j) if (j < k) racc -= alpha[j] * mv[j];
            }
        } else {
            for (int i = tid; i < m; i += NT) {
                float s = yv[i];
                for (int j = 0; j < k; ++j) s -= alpha[j] * p.Mr[(size_t)i * N + selcol[j]];
                rv[i] = s;
            }
            __syncthreads();
        }
        // g = M_S^T r
        if (one_row) {
            const int mwaves = (m + 63) >> 6;
            if (wave < mwaves) {
#pragma unroll
                for (int j = 0; j < RF_MAXK; ++j) {
                    if (j < k) {                           // k is uniform: no divergence
                        const float s = wave_sum(tid < m ? mv[j] * racc : 0.f);
                        if (lane == 0) gv[wave * RF_MAXK + j] = s;
                    }
                }
            }
            __syncthreads();
            if (wave == 0 && lane < k) {
                float s = 0.f;
                for (int q = 0; q < mwaves; ++q) s += gv[q * RF_MAXK + lane];
                gv[lane] = s;
            }
        } else {
            for (int j = wave; j < k; j += nwaves) {
                float s = 0.f;
                for (int i = lane; i < m; i += 64) s += p.Mr[(size_t)i * N + selcol[j]] * rv[i];
                s = wave_sum(s);
                if (lane == 0) gv[j] = s;
            }
            __syncthreads();
        }
        // one refinement step: (R^T R) delta = g
        if (wave == 0) {
            const float wv = solve_lower_t(lane < k ? gv[lane] : 0.f);
            const float dl = solve_upper(wv);
            if (lane < k) { alpha[lane] += dl; beta[lane] = dl; }
        }
        __syncthreads();
        float ss = 0.f;
        if (one_row) {
            if (tid < m) {
#pragma unroll
                for (int j = 0; j < RF_MAXK; ++j) if (j < k) racc -= beta[j] * mv[j];
                ss = racc * racc;
            }
        } else {
            for (int i = tid; i < m; i += NT) {
                float s = rv[i];
                for (int j = 0; j < k; ++j) s -= beta[j] * p.Mr[(size_t)i * N + selcol[j]];
                ss += s * s;
            }
        }
        ss = wave_sum(ss);
        if (lane == 0) red[wave] = ss;
        __syncthreads();
    }
    if (WANT_FIT) {
        for (int qi = tid; qi < k; qi += NT) {
            const int g = selcol[qi];
            int rank = 0;
            for (int o = 0; o < k; ++o) rank += selcol[o] < g;
            a.support[(size_t)prob * k + rank] = g;
            if (a.coef) a.coef[(size_t)prob * k + rank] = alpha[qi];
        }
    } else {
        // ascending support straight from the selection flags: the rank of a selected atom is the number
        // of selected atoms below it (no record of the order of selection is kept in this variant)
        const unsigned long long sb = __ballot(selected);
        if (lane == 0) red[wave] = __int_as_float(__popcll(sb));
        __syncthreads();
        if (selected) {
            int rank = __popcll(sb & ((1ull << lane) - 1ull));
            for (int wv = 0; wv < wave; ++wv) rank += __float_as_int(red[wv]);
            a.support[(size_t)prob * k + rank] = tid;
        }
    }
    if (tid == 0) {
        if (a.resid) {
            float tot = 0.f;
            for (int wv = 0; wv < nwaves; ++wv) tot += red[wv];
            a.resid[prob] = bad ? __int_as_float(0x7fc00000) : sqrtf(tot);
        }
        if (WANT_MARGIN) a.margin[prob] = bad ? 0.f : margin;   // every round wave tracked the same value
    }
}

// ---------------------------------------------------------------------------
// Two sketches per workgroup, for launches with more problems than the chip has compute units (the decode
// loop's batched call: tokens x layers).  The rounds of recover_fast_kernel keep three waves of a
// workgroup busy at the 7B FFN shape and a compute unit holds one such workgroup (the Gram matrix fills its
// LDS), so 512 problems take two turns.  Here two tokens of the same operator share one copy of the Gram
// matrix, stored as its lower triangle (it is symmetric entry by entry: both halves are the same sum of the
// same products in the same order), each with a group of waves, a factor and a candidate area of its own;
// the per-token arithmetic is that of recover_fast_kernel<true, *, false>, operation by operation, so the
// supports and margins are the same bits.  M is read once for the two tokens.
// ---------------------------------------------------------------------------
struct PairLayout {
    int group_floats;     // per token: off_y .. end of the factor
    int off_y, off_cand, off_red, off_Dt;
    int off_tri;          // the Gram triangle, after the two groups
    int KS, total_floats;
};

static bool make_pair_layout(const Plan& p, int k, int lds_limit, PairLayout& L) {
    const int N = p.N, m = p.op.m;
    int ks = (k + 3) & ~3;
    if (((ks >> 2) & 1) == 0) ks += 4;        // an odd number of 16-byte groups per row, as in the single-token layout
    L.KS = ks;
    int o = 0;
    L.off_y = o; o += (m + 3) & ~3;
    L.off_cand = o; o += 2 * 16 * 8;
    L.off_red = o; o += 16;
    int dt = N * ks;
    if (dt < RF_THREADS * 4) dt = RF_THREADS * 4;          // doubles as the staging area of the first correlations
    L.off_Dt = o; o += (dt + 3) & ~3;
    L.group_floats = o;
    L.off_tri = 2 * o;
    const long total = 2L * o + (long)N * (N + 1) / 2;
    L.total_floats = (int)total;
    return total <= lds_limit / 4 - 16;
}

template <bool WANT_MARGIN>
__global__ __launch_bounds__(RF_THREADS)
void recover_pair_kernel(Plan p, RecoverArgs a, PairLayout L) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x;
    constexpr int NT = RF_THREADS;
    const int lane = tid & 63, wave = tid >> 6;
    if (a.plans) p = a.plans[blockIdx.y];
    const int N = p.N, m = p.op.m, k = a.k, KS = L.KS;
    const int round_waves = (N + 63) >> 6;     // waves per token in the rounds; the host checks 2 * round_waves <= NT / 64
    const int grp = wave / round_waves;        // the token this wave serves in the rounds (2 and above: none)
    const int lw = wave - grp * round_waves;   // the wave's place in its group
    const int c = tid - grp * round_waves * 64;   // atom of this thread in the rounds
    const bool in_group = grp < 2;
    const bool active = in_group && c < N;
    const int t0 = 2 * blockIdx.x;
    const int ntok = min(2, a.B - t0);         // a lone last token is solved twice and stored once
    const int prob0 = blockIdx.y * a.B + t0, prob1 = prob0 + (ntok == 2 ? 1 : 0);

    float* base0 = lds, * base1 = lds + L.group_floats;
    float* mine = in_group && grp == 1 ? base1 : base0;
    float* yv0 = base0 + L.off_y, * yv1 = base1 + L.off_y;
    float* cand = mine + L.off_cand;           // [2][16][8]
    float* red = mine + L.off_red;
    float* Dt = mine + L.off_Dt;               // [N][KS], row c = factor entries of atom c
    float* tri = lds + L.off_tri;              // G[i][j], j <= i, at i (i + 1) / 2 + j

    // ---- every independent global load is issued before the first wait
    const float* y0 = a.y + (size_t)prob0 * m, * y1 = a.y + (size_t)prob1 * m;
    const float yreg0 = (tid < m) ? y0[tid] : 0.f, yreg1 = (tid < m) ? y1[tid] : 0.f;
    const float w = (active && p.weighted) ? p.W[c] : 1.f;
    const float gd = active ? p.gram[(size_t)c * N + c] : 1.f;
    constexpr int GU = 8;
    const int n4 = (N * N) >> 2;               // N is a multiple of 4: a group of four never straddles rows
    const float4* gsrc = reinterpret_cast<const float4*>(p.gram);
    float4 greg[GU];
    int grow_[GU], gcol_[GU];
    auto row_col = [&](int idx, int& row, int& col) {
        // (4 idx) / N without the integer division: exact, 4 idx < 2^18 and N <= 256 keep (4 idx + 0.5) / N
        // further than 2^-10 from the next integer
        row = (int)__fdividef((float)(4 * idx) + 0.5f, (float)N);
        col = 4 * idx - row * N;
    };
#pragma unroll
    for (int u = 0; u < GU; ++u) {
        const int idx = u * NT + tid;
        row_col(idx, grow_[u], gcol_[u]);
        const bool need = idx < n4 && gcol_[u] <= grow_[u];
        greg[u] = need ? gsrc[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
        if (!need) grow_[u] = -1;
    }
    auto to_tri = [&](const float4& v, int row, int col) {
        float* dst = tri + (row * (row + 1)) / 2 + col;
        dst[0] = v.x;
        if (col + 1 <= row) dst[1] = v.y;
        if (col + 2 <= row) dst[2] = v.z;
        if (col + 3 <= row) dst[3] = v.w;
    };
    // slices of M^T y: a thread takes four adjacent atoms and a contiguous range of rows, for both tokens
    const int ncg = N >> 2;
    const int parts = NT / ncg;
    const int cg = tid % ncg, part = tid / ncg;
    const int rows_per = (m + parts - 1) / parts;
    const int i0 = part * rows_per, i1 = part < parts ? min(m, i0 + rows_per) : i0;
    constexpr int MU = 8;
    float4 mreg[MU];
    const float4* mr = reinterpret_cast<const float4*>(p.Mr) + cg;
#pragma unroll
    for (int u = 0; u < MU; ++u)
        mreg[u] = (i0 + u < i1) ? mr[(size_t)(i0 + u) * ncg] : make_float4(0.f, 0.f, 0.f, 0.f);
    int bad0 = !isfinite(yreg0), bad1 = !isfinite(yreg1);
    if (tid < m) { yv0[tid] = yreg0; yv1[tid] = yreg1; }
    for (int i = tid + NT; i < m; i += NT) {          // only when m exceeds the workgroup size
        const float v0 = y0[i], v1 = y1[i];
        yv0[i] = v0; yv1[i] = v1;
        if (!isfinite(v0)) bad0 = 1;
        if (!isfinite(v1)) bad1 = 1;
    }
#pragma unroll
    for (int u = 0; u < GU; ++u) if (grow_[u] >= 0) to_tri(greg[u], grow_[u], gcol_[u]);
    for (int base = GU * NT; base < n4; base += NT) {
        const int idx = base + tid;
        int row, col;
        row_col(idx, row, col);
        if (idx < n4 && col <= row) to_tri(gsrc[idx], row, col);
    }
    bad0 = __syncthreads_or(bad0);
    bad1 = __syncthreads_or(bad1);

    float corr = 0.f;
    {
        float* stage0 = base0 + L.off_Dt, * stage1 = base1 + L.off_Dt;     // [parts][N] each
        float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
        for (int ib = i0; ib < i1; ib += MU) {
            if (ib != i0) {
#pragma unroll
                for (int u = 0; u < MU; ++u)
                    mreg[u] = (ib + u < i1) ? mr[(size_t)(ib + u) * ncg] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < MU; ++u)
                if (ib + u < i1) {
                    const float ya = yv0[ib + u], yb = yv1[ib + u];
                    acc0.x += mreg[u].x * ya; acc0.y += mreg[u].y * ya; acc0.z += mreg[u].z * ya; acc0.w += mreg[u].w * ya;
                    acc1.x += mreg[u].x * yb; acc1.y += mreg[u].y * yb; acc1.z += mreg[u].z * yb; acc1.w += mreg[u].w * yb;
                }
        }
        if (part < parts) {
            reinterpret_cast<float4*>(stage0)[part * ncg + cg] = acc0;
            reinterpret_cast<float4*>(stage1)[part * ncg + cg] = acc1;
        }
        __syncthreads();
        if (active) for (int q = 0; q < parts; ++q) corr += Dt[q * N + c];
        __syncthreads();                                // the staging areas become the factors
    }
    bool selected = false;
    float margin = 1.f;
    float sq = 0.f;                                     // squared norm of the thread's factor row so far
    float* myrow = Dt + (size_t)(active ? c : 0) * KS;
    // rows are zero beyond their last written entry, so that a round may read whole groups of four
    for (int i = tid; i < (N * KS) >> 2; i += NT) {
        reinterpret_cast<float4*>(base0 + L.off_Dt)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        reinterpret_cast<float4*>(base1 + L.off_Dt)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    int badr = 0;
    for (int J = 0; J < k; ++J) {
        if (in_group) {
            // key: 0 for lanes without a candidate, else 1 + the bit pattern of the (non-negative) score
            uint32_t key = 0u;
            if (active && !selected) {
                const float t = w * corr;
                float score = t * t;
                if (!(score >= 0.f)) score = 0.f;        // NaN scores tie at zero
                key = __float_as_uint(score) + 1u;
            }
            const uint32_t m1 = wave_max_u32(key);
            const unsigned long long hit = __ballot(key == m1);
            const int l1 = __ffsll((long long)hit) - 1;
            const float c1 = readlane_f32(corr, l1);
            const float nrm2 = gd - sq;
            float rs = 0.f;
            if (nrm2 > 1e-10f * gd && nrm2 > 0.f) rs = __builtin_amdgcn_rsqf(nrm2);
            const float i1v = readlane_f32(rs, l1);
            uint32_t m2 = 0u;
            if (WANT_MARGIN) m2 = wave_max_u32(lane == l1 ? 0u : key);
            if (lane == 0) {
                float4 cv;
                cv.x = __uint_as_float(m1); cv.y = __int_as_float(lw * 64 + l1); cv.z = __uint_as_float(m2); cv.w = c1;
                float* cw = cand + ((J & 1) * 16 + lw) * 8;
                *reinterpret_cast<float4*>(cw) = cv;
                cw[4] = i1v;
            }
        }
        __syncthreads();
        if (in_group) {
            const float* cb = cand + (J & 1) * 16 * 8;
            uint32_t k1 = 0u, k2 = 0u;
            int gstar = 0;
            float ccol = 0.f, inv = 0.f;
            for (int w0 = 0; w0 < round_waves; w0 += 4) {
                float4 cw[4];
                float ci[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (w0 + q < round_waves) {
                        const float* e = cb + (w0 + q) * 8;
                        cw[q] = *reinterpret_cast<const float4*>(e);
                        ci[q] = e[4];
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (w0 + q >= round_waves) break;
                    const uint32_t o1 = __float_as_uint(cw[q].x);
                    const uint32_t o2 = __float_as_uint(cw[q].z);
                    const bool up = o1 > k1 || w0 + q == 0;   // ties keep the lower wave = lower index
                    k2 = up ? max(max(k2, k1), o2) : max(k2, o1);
                    gstar = up ? __float_as_int(cw[q].y) : gstar;
                    ccol = up ? cw[q].w : ccol;
                    inv = up ? ci[q] : inv;
                    k1 = up ? o1 : k1;
                }
            }
            if (WANT_MARGIN) {
                const float s1 = __uint_as_float(k1 - 1u);
                const float s2 = k2 ? __uint_as_float(k2 - 1u) : 0.f;
                margin = fminf(margin, s1 > 0.f ? (s1 - s2) * __builtin_amdgcn_rcpf(s1) : 0.f);
            }
            if (c == gstar) selected = true;
            const int hi = max(gstar, c), lo = min(gstar, c);
            const float gmine = active ? tri[(hi * (hi + 1)) / 2 + lo] : 0.f;
            const float* prow = Dt + (size_t)gstar * KS;
            float dot = 0.f;
            const int JU = (J + 3) & ~3;               // whole groups of four: the rows end in zeros
            int j = 0;
            for (; j + 16 <= JU; j += 16) {
                float4 u[4], v[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u[q] = *reinterpret_cast<const float4*>(myrow + j + 4 * q);
                    v[q] = *reinterpret_cast<const float4*>(prow + j + 4 * q);
                }
                float d2 = 0.f;
#pragma unroll
                for (int q = 0; q < 4; q += 2) {
                    dot += u[q].x * v[q].x + u[q].y * v[q].y + u[q].z * v[q].z + u[q].w * v[q].w;
                    d2 += u[q + 1].x * v[q + 1].x + u[q + 1].y * v[q + 1].y + u[q + 1].z * v[q + 1].z + u[q + 1].w * v[q + 1].w;
                }
                dot += d2;
            }
            if (j < JU) {
                const float4 u0 = *reinterpret_cast<const float4*>(myrow + j);
                const float4 v0 = *reinterpret_cast<const float4*>(prow + j);
                if (j + 4 < JU) {
                    const float4 u1 = *reinterpret_cast<const float4*>(myrow + j + 4);
                    const float4 v1 = *reinterpret_cast<const float4*>(prow + j + 4);
                    if (j + 8 < JU) {
                        const float4 u2 = *reinterpret_cast<const float4*>(myrow + j + 8);
                        const float4 v2 = *reinterpret_cast<const float4*>(prow + j + 8);
                        dot += u2.x * v2.x + u2.y * v2.y + u2.z * v2.z + u2.w * v2.w;
                    }
                    dot += u1.x * v1.x + u1.y * v1.y + u1.z * v1.z + u1.w * v1.w;
                }
                dot += u0.x * v0.x + u0.y * v0.y + u0.z * v0.z + u0.w * v0.w;
            }
            if (inv == 0.f) badr = 1;
            const float dv = (gmine - dot) * inv;
            const float bt = ccol * inv;
            corr -= bt * dv;
            sq += dv * dv;
            if (active) myrow[J] = dv;
        }
    }
    bad0 = __syncthreads_or(bad0 | (grp == 0 ? badr : 0));
    bad1 = __syncthreads_or(bad1 | (grp == 1 ? badr : 0));

    // ascending support straight from the selection flags: the rank of a selected atom is the number of
    // selected atoms below it
    const unsigned long long sb = __ballot(selected);
    if (in_group && lane == 0) red[lw] = __int_as_float(__popcll(sb));
    __syncthreads();
    const bool stores = in_group && grp < ntok;
    const int prob = grp == 1 ? prob1 : prob0;
    if (stores && selected) {
        int rank = __popcll(sb & ((1ull << lane) - 1ull));
        for (int wv = 0; wv < lw; ++wv) rank += __float_as_int(red[wv]);
        a.support[(size_t)prob * k + rank] = c;
    }
    if (WANT_MARGIN && stores && lw == 0 && lane == 0) a.margin[prob] = (grp == 1 ? bad1 : bad0) ? 0.f : margin;
}

template <bool WANT_MARGIN>
static hipError_t launch_pair(const Plan& p, const RecoverArgs& a, const PairLayout& PL, hipStream_t s) {
    const size_t bytes = (size_t)PL.total_floats * 4;
    static size_t allowed = 0;
    if (bytes > allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_pair_kernel<WANT_MARGIN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        allowed = bytes;
    }
    hipLaunchKernelGGL((recover_pair_kernel<WANT_MARGIN>), dim3((a.B + 1) / 2, a.nplans), dim3(RF_THREADS), bytes, s, p, a, PL);
    return hipGetLastError();
}

template <bool GRAM_LDS, bool WANT_MARGIN, bool WANT_FIT>
static hipError_t launch_fast(const Plan& p, const RecoverArgs& a, const FastLayout& FL, int nthreads, hipStream_t s) {
    const size_t bytes = (size_t)FL.total_floats * 4;
    static size_t allowed = 0;              // raise the dynamic LDS limit only when a launch needs more
    if (bytes > allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_fast_kernel<GRAM_LDS, WANT_MARGIN, WANT_FIT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        allowed = bytes;
    }
    hipLaunchKernelGGL((recover_fast_kernel<GRAM_LDS, WANT_MARGIN, WANT_FIT>), dim3(a.B, a.nplans), dim3(nthreads), bytes, s, p, a, FL);
    return hipGetLastError();
}

hipError_t launch_recover(const Plan& p, const RecoverArgs& a, int lds_limit, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    const bool fit = a.coef != nullptr || a.resid != nullptr;
    if (p.rb == 1 && p.N <= RF_THREADS && a.k <= (fit ? RF_MAXK : RF_MAXK_SELECT)) {
        // one wavefront for small problems, otherwise a full workgroup so that the bulk loads
        // (Gram matrix, M) have many requests in flight
        const int nthreads = (p.N <= 64 && p.op.m <= 64) ? 64 : RF_THREADS;
        // more problems than compute units, supports only: two tokens of an operator per workgroup
        PairLayout PL;
        if (!fit && nthreads == RF_THREADS && a.B >= 2 && (long)a.B * a.nplans > RP_MIN_PROBLEMS && (p.N & 3) == 0 &&
            2 * ((p.N + 63) / 64) <= RF_THREADS / 64 && make_pair_layout(p, a.k, lds_limit, PL))
            return a.margin ? launch_pair<true>(p, a, PL, s) : launch_pair<false>(p, a, PL, s);
        FastLayout FL;
        if (make_fast_layout(p, a.k, lds_limit, nthreads, fit, a.spill != nullptr && a.spill_stride >= (size_t)a.k * p.N, FL)) {
            const bool gl = FL.off_gram >= 0, mg = a.margin != nullptr;
#define CS_RF(G_, M_) (fit ? launch_fast<G_, M_, true>(p, a, FL, nthreads, s) : launch_fast<G_, M_, false>(p, a, FL, nthreads, s))
            if (gl && mg) return CS_RF(true, true);
            if (gl && !mg) return CS_RF(true, false);
            if (!gl && mg) return CS_RF(false, true);
            return CS_RF(false, false);
#undef CS_RF
        }
    }
    const RecoverLayout L = make_layout(p, a.k, lds_limit);
    int nt = 256;
    if (p.N > 256) nt = 512;
    if (p.N > 512) nt = 1024;
    const size_t bytes = (size_t)L.total_floats * 4;
    static size_t allowed = 0;
    if (bytes > allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e != hipSuccess) return e;
        allowed = bytes;
    }
    hipLaunchKernelGGL(recover_kernel, dim3(a.B, a.nplans), dim3(nt), bytes, s, p, a, L);
    return hipGetLastError();
}

}  // namespace csk
