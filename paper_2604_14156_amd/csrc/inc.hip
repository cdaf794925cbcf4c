// Warm-started structured recovery: the previous token's support is corrected by a
// backward/forward exchange instead of being recovered from nothing (paper Sec. 5: temporal
// regulariser gamma ||alpha_t - alpha_{t-1}||^2 and incremental support updates; Sec. 10,
// proposition on incremental token-adaptive recovery).  One workgroup per sketch, one atom
// per unit.
//
//   1. alpha1 = argmin ||y - M_S a||^2 + gamma ||a - alpha_prev||^2 on the previous support S;
//   2. the `swaps` units of S with the least energy (alpha1_j ||m_j||)^2 leave (among equal
//      energies the larger index first);
//   3. `swaps` greedy rounds (score of the unselected units on the residual of the least-squares
//      fit of the current units, ties -> smaller index) bring the support back to k units;
//   4. least-squares refit, explicit residual, one refinement step.
//
// Everything runs in the Gram domain (G = M^T M in LDS, c0 = M^T y): the correlation with the
// residual of a fit on S is c0 - G[:, S] alpha, the fits are Cholesky solves of G_SS by one
// wavefront (a factorisation per refit of a changed list, one appended row per greedy round).
#include "kernels.hpp"
#include "common.hpp"
#include "small_dense.hpp"
#include "gram_loads.hpp"

namespace csk {

constexpr int IN_MAXK = 64;
constexpr int IN_THREADS = 512;

struct IncLayout {
    int off_y, off_r, off_c0, off_nrm, off_flag, off_S, off_S2, off_t, off_L, off_misc, off_red, off_gram, off_stage;
    int total_floats;
};

static bool make_inc_layout(const Plan& p, int lds_limit, int nthreads, IncLayout& L, bool want_gram = true) {
    const int N = p.N, m = p.op.m;
    const int Np = (N + 7) & ~7;
    int o = 0;
    L.off_y = o; o += (m + 3) & ~3;
    L.off_r = o; o += (m + 3) & ~3;
    L.off_c0 = o; o += Np;
    L.off_nrm = o; o += Np;
    L.off_flag = o; o += Np;
    L.off_S = o; o += IN_MAXK;
    L.off_S2 = o; o += IN_MAXK;
    L.off_t = o; o += 4 * IN_MAXK;
    L.off_L = o; o += IN_MAXK * (IN_MAXK + 4);      // factor (row stride 65) or carried inverse (row stride 68)
    L.off_misc = o; o += 32;
    L.off_red = o; o += 64;                  // per wave: 64-bit best key, runner-up score
    L.off_stage = o; o += nthreads * 4;
    L.off_gram = -1;
    const long limit = lds_limit / 4 - 16;
    if (o > limit) return false;
    if (want_gram && (long)o + (long)N * N <= limit) { L.off_gram = o; o += N * N; }
    L.total_floats = o;
    return true;
}

template <bool GRAM_LDS>
__global__ __launch_bounds__(IN_THREADS)
void recover_inc_kernel(Plan p, RecoverArgs a, IncArgs q, IncLayout L) {
    extern __shared__ float lds[];
    const int tid = threadIdx.x, NT = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = NT >> 6;
    const int prob = blockIdx.x;
    const int N = p.N, m = p.op.m, k = a.k;
    const int swaps = q.swaps, K0 = k - swaps;
    const bool active = tid < N;

    float* yv = lds + L.off_y;
    float* rv = lds + L.off_r;
    float* c0v = lds + L.off_c0;
    float* nrm = lds + L.off_nrm;
    int* flag = reinterpret_cast<int*>(lds + L.off_flag);
    int* S = reinterpret_cast<int*>(lds + L.off_S);
    int* S2 = reinterpret_cast<int*>(lds + L.off_S2);
    float* tv = lds + L.off_t;                  // [4][IN_MAXK] small vectors
    float* Lf = lds + L.off_L;                  // Cholesky factor, row stride IN_MAXK + 1
    int* misc = reinterpret_cast<int*>(lds + L.off_misc);
    float* red = lds + L.off_red;
    float* stage = lds + L.off_stage;
    float* gram_l = lds + L.off_gram;
    const float* gram = GRAM_LDS ? gram_l : p.gram;
    float* beta = tv, *xs = tv + IN_MAXK, *gv = tv + 2 * IN_MAXK, *dl = tv + 3 * IN_MAXK;

    // ---- loads: sketch, atom norms, Gram matrix, c0 = M^T y
    const float* y = a.y + (size_t)prob * m;
    int bad = 0;
    float iw = 1.f, w = 1.f;                           // W holds 1/norm of the atom
    if (active && p.weighted) { iw = p.W[tid]; w = iw > 0.f ? 1.0f / iw : 0.f; }
    if (active) { nrm[tid] = w; flag[tid] = 0; }
    // previous support: in range and without repeats, else the row is reported as failed
    if (wave == 0) {
        const int u = lane < k ? q.prev_support[(size_t)prob * k + lane] : -1;
        int ok = lane >= k || (u >= 0 && u < p.G);
        for (int i = 0; i < k; ++i) {
            const int ui = __builtin_amdgcn_readlane(u, i);
            if (lane < k && lane != i && ui == u) ok = 0;
        }
        if (!ok) bad = 1;
        if (lane < k) S[lane] = ok ? u : 0;
    }
    const float c0 = load_sketch_gram_c0<GRAM_LDS>(p, y, yv, gram_l, stage, bad);
    if (active) c0v[tid] = c0;
    __syncthreads();
    if (bad) {                                           // uniform: NaN sketch or invalid previous support
        for (int i = tid; i < k; i += NT) {
            a.support[(size_t)prob * k + i] = -1;
            if (a.coef) a.coef[(size_t)prob * k + i] = 0.f;
        }
        if (tid == 0) {
            if (a.resid) a.resid[prob] = __int_as_float(0x7fc00000);
            if (a.margin) a.margin[prob] = 0.f;
        }
        return;
    }

    // ---- 1./2. regularised refit on the previous support, then the backward step.
    // The list is first put in the order of a cheap proxy of the unit energies (matched filter,
    // strongest first).  The units that leave are decided by the energies of the fit itself; when
    // they turn out to be the last `swaps` of that order (the usual case) the leading part of the
    // factor and of the forward-substituted right-hand side is already the fit of the kept units.
    const bool ridge = q.prev_coef != nullptr && q.gamma > 0.f;
    float zreg = 0.f;                                  // wave 0, lane j: component j of L^{-1} c0_S
    if (wave == 0 && swaps == k && lane == 0) misc[0] = 0;   // everything leaves: nothing to fit
    if (wave == 0 && swaps < k) {
        const int u = lane < k ? S[lane] : 0x7fffffff;
        float pcoef = (ridge && lane < k) ? q.prev_coef[(size_t)prob * k + lane] : 0.f;
        // rank by (value descending, unit index ascending) within the first k lanes
        auto rank_of = [&](float e) -> int {
            int rank = 0;
            for (int i = 0; i < k; ++i) {
                const float ei = readlane_f32(e, i);
                const int ui = __builtin_amdgcn_readlane(u, i);
                rank += (int)(ei > e) | ((int)(ei == e) & (int)(ui < u));
            }
            return rank;
        };
        int pos = lane;                                  // position of this lane's unit in the list
        if (swaps > 0) {
            float pe = lane < k ? c0v[lane < k ? u : 0] * (p.weighted ? p.W[lane < k ? u : 0] : 1.f) : -1.f;
            pe = pe * pe;
            if (lane >= k) pe = -1.f; else if (!(pe >= 0.f)) pe = 0.f;
            pos = rank_of(pe);
            __builtin_amdgcn_wave_barrier();
            if (lane < k) { S[pos] = u; xs[pos] = pcoef; }
            __builtin_amdgcn_wave_barrier();
            pcoef = lane < k ? xs[lane] : 0.f;           // previous coefficient of the unit now at `lane`
        }
        const int su = lane < k ? S[lane] : 0x7fffffff;   // unit at position `lane`
        int wbad = wave_cholesky(gram, N, S, k, ridge ? q.gamma : 0.f, Lf, gv, lane);
        float rhs = lane < k ? c0v[su] : 0.f;
        if (ridge) rhs += q.gamma * pcoef;
        zreg = wave_forward(Lf, k, rhs, lane);
        const float x = wave_backward(Lf, k, zreg, lane);
        if (swaps == 0) {
            if (lane < k) xs[lane] = x;
            if (ridge) {                                 // the fit reported is the plain one: factor without the ridge
                wbad |= wave_cholesky(gram, N, S, k, 0.f, Lf, gv, lane);
                const float x0 = wave_cholesky_solve(Lf, k, lane < k ? c0v[su] : 0.f, lane);
                if (lane < k) xs[lane] = x0;
            }
        } else {
            // energies of the fit decide; same ordering rule, now on the reordered list
            float e = lane < k ? x * nrm[lane < k ? su : 0] : -1.f;
            e = e * e;
            if (lane >= k) e = -1.f; else if (!(e >= 0.f)) e = 0.f;
            int rank = 0;                                // 0 = strongest; equal energies: smaller index first
            for (int i = 0; i < k; ++i) {
                const float ei = readlane_f32(e, i);
                const int ui = __builtin_amdgcn_readlane(su, i);
                rank += (int)(ei > e) | ((int)(ei == e) & (int)(ui < su));
            }
            const bool keep = lane < k && rank < K0;
            const bool agrees = lane >= k || (keep == (lane < K0));
            const bool reuse = !ridge && __ballot(!agrees) == 0ull;
            if (reuse) {
                const float xk = wave_backward(Lf, K0, zreg, lane);
                if (lane < K0) xs[lane] = xk;
            } else {
                __builtin_amdgcn_wave_barrier();
                if (keep) S[rank] = su;                  // kept units to the front (every lane has read its unit)
                __builtin_amdgcn_wave_barrier();
                if (K0 > 0) wbad |= wave_cholesky(gram, N, S, K0, 0.f, Lf, gv, lane);
                zreg = wave_forward(Lf, K0, lane < K0 ? c0v[S[lane]] : 0.f, lane);
                const float xk = wave_backward(Lf, K0, zreg, lane);
                if (lane < K0) xs[lane] = xk;
            }
        }
        if (lane == 0) misc[0] = wbad;
    }
    __syncthreads();
    if (tid < K0) flag[S[tid]] = 1;
    __syncthreads();

    // ---- 3. forward step
    float margin = 1.f;
    unsigned long long* redk = reinterpret_cast<unsigned long long*>(red);       // [nwaves] best keys
    float* red2 = red + 32;                                                       // [nwaves] runner-up scores
    for (int it = 0; it < swaps; ++it) {
        const int K = K0 + it;
        // correlation with the residual of the current fit: c0 - G[:, S] alpha.  Every wave keeps the
        // list and its coefficients in its first K lanes and hands them out by scalar lane reads.
        const int sreg = lane < K ? S[lane] : 0;
        const float areg = lane < K ? xs[lane] : 0.f;
        const int ta = active ? tid : 0;
        float acc = 0.f;
        for (int j = 0; j < K; j += 4) {
            float gv4[4], av4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {               // lanes >= K hold index 0 and coefficient 0; j + u <= 63
                const int sj = __builtin_amdgcn_readlane(sreg, j + u);
                av4[u] = readlane_f32(areg, j + u);
                gv4[u] = gram[(size_t)sj * N + ta];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc += av4[u] * gv4[u];
        }
        float sc = iw * (c0 - acc);
        sc = sc * sc;
        if (!(sc >= 0.f)) sc = 0.f;
        const bool cand = active && flag[tid] == 0;
        // best (ties -> smaller index) and runner-up: keys order by score, then by descending index
        unsigned long long key = cand ? ((unsigned long long)__float_as_uint(sc) << 32) | (0xffffffffu - (unsigned)tid) : 0ull;
        unsigned long long kb = key;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long o = __shfl_xor(kb, off);
            kb = o > kb ? o : kb;
        }
        const float s2w = wave_max(cand && key != kb ? sc : -1.f);
        if (lane == 0) { redk[wave] = kb; red2[wave] = s2w; }
        __syncthreads();
        unsigned long long gb = 0ull;
        for (int wv = 0; wv < nwaves; ++wv) { const unsigned long long o = redk[wv]; gb = o > gb ? o : gb; }
        float s2 = 0.f;
        for (int wv = 0; wv < nwaves; ++wv) {
            const unsigned long long o = redk[wv];
            if (o != gb && o != 0ull) s2 = fmaxf(s2, __uint_as_float((unsigned)(o >> 32)));
            s2 = fmaxf(s2, red2[wv]);
        }
        const float s1 = __uint_as_float((unsigned)(gb >> 32));
        const int best = min(max((int)(0xffffffffu - (unsigned)(gb & 0xffffffffull)), 0), N - 1);   // always a candidate: K < k <= N
        margin = fminf(margin, s1 > 0.f ? (s1 - s2) / s1 : 0.f);
        if (wave == 0) {
            // new row of the factor, new last component of L^{-1} c0_S, then only the backward substitution
            float lrow = 0.f;
            const int wbad = wave_cholesky_append(gram, N, S, K, best, Lf, lane, &lrow);
            const float dot = wave_sum(lane < K ? lrow * zreg : 0.f);
            const float zk = (c0v[best] - dot) * Lf[K * SD_LS + SD_MAXK];
            if (lane == K) zreg = zk;
            if (lane == 0) { S[K] = best; flag[best] = 1; if (wbad) misc[0] = 1; }
            const float x = wave_backward(Lf, K + 1, zreg, lane);
            if (lane <= K) xs[lane] = x;
        }
        __syncthreads();
    }
    bad = misc[0];

    // ---- 4. explicit residual and one refinement step on the final support
    const bool want_fit = a.coef != nullptr || a.resid != nullptr;
    if (want_fit) {
        for (int i = tid; i < m; i += NT) {
            float s = yv[i];
            for (int j = 0; j < k; ++j) s -= xs[j] * p.Mr[(size_t)i * N + S[j]];
            rv[i] = s;
        }
        __syncthreads();
        for (int j = wave; j < k; j += nwaves) {
            float s = 0.f;
            for (int i = lane; i < m; i += 64) s += p.Mr[(size_t)i * N + S[j]] * rv[i];
            s = wave_sum(s);
            if (lane == 0) gv[j] = s;
        }
        __syncthreads();
        if (wave == 0) {
            const float d = wave_cholesky_solve(Lf, k, lane < k ? gv[lane] : 0.f, lane);
            if (lane < k) { xs[lane] += d; dl[lane] = d; }
        }
        __syncthreads();
        float ss = 0.f;
        for (int i = tid; i < m; i += NT) {
            float s = rv[i];
            for (int j = 0; j < k; ++j) s -= dl[j] * p.Mr[(size_t)i * N + S[j]];
            ss += s * s;
        }
        ss = wave_sum(ss);
        if (lane == 0) beta[wave] = ss;                  // beta[] is free: per-wave partial sums
        __syncthreads();
    }
    for (int qi = tid; qi < k; qi += NT) {
        const int gsel = S[qi];
        int rank = 0;
        for (int o = 0; o < k; ++o) rank += S[o] < gsel;
        a.support[(size_t)prob * k + rank] = gsel;
        if (a.coef) a.coef[(size_t)prob * k + rank] = xs[qi];
    }
    if (tid == 0) {
        if (a.resid) {
            float tot = 0.f;
            for (int wv = 0; wv < nwaves; ++wv) tot += beta[wv];
            a.resid[prob] = bad ? __int_as_float(0x7fc00000) : sqrtf(tot);
        }
        if (a.margin) a.margin[prob] = bad ? 0.f : margin;
    }
}

// ---------------------------------------------------------------------------------------------
// The same exchange with state carried from token to token (Sec. 5: the loop runs once per token and
// the support drifts slowly; Sec. 10: only the changed part has to be identified).  What a token
// leaves behind is the inverse of the Gram matrix of its support, P = (G_SS)^{-1}, with the order of
// its units; the next token's work on that support is then
//     fit:     alpha = P c0_S                                     (one k x k product)
//     leave:   P' = P_{-j,-j} - P_{-j,j} P_{j,-j} / P_jj           (unit at position j removed)
//     enter:   w = P g, s = G_uu - g^T w,  P' = [P + w w^T / s, -w / s; -w^T / s, 1 / s]   (g = G_{S,u})
// all of them k^2 multiply-adds without a dependent chain, against a factorisation (k^3 / 6 in a chain of
// k steps) per changed list in the kernel above.  Rounding errors of the updates add up from token to
// token, so the inverse is built again from nothing every IN_REFRESH tokens, and whenever the caller's
// previous support is not the set the state was left for.  No ridge term: the carried inverse is that of
// G_SS itself.
//
// P lives in the LDS area of the factor; wavefront 0 owns it, lane i = row i.
constexpr int IN_REFRESH = 64;
constexpr uint32_t IN_MAGIC = 0x43530000u;

__device__ __forceinline__ void inc_wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Row stride of P: a multiple of four floats, so that rows are read and written 16 bytes at a time, and
// 4 mod 64, so that the 16-byte accesses of 16 consecutive lanes fall into different banks.  Everything of
// the 64 x 64 area outside the leading K x K block is kept at zero, and so are the vectors beyond K: the
// loops below run to the next multiple of four without masks.
constexpr int IN_PS = IN_MAXK + 4;

// row[j] += c * v[j] for j < K rounded up to 4 (row: this lane's row of P; v in LDS, zero beyond K)
__device__ __forceinline__ void inv_row_axpy(float* row, int K, float c, const float* v) {
    for (int j0 = 0; j0 < K; j0 += 8) {
        float4 r0 = *reinterpret_cast<const float4*>(row + j0), v0 = *reinterpret_cast<const float4*>(v + j0);
        const bool two = j0 + 4 < K;
        float4 r1 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = r1;
        if (two) { r1 = *reinterpret_cast<const float4*>(row + j0 + 4); v1 = *reinterpret_cast<const float4*>(v + j0 + 4); }
        r0.x += c * v0.x; r0.y += c * v0.y; r0.z += c * v0.z; r0.w += c * v0.w;
        r1.x += c * v1.x; r1.y += c * v1.y; r1.z += c * v1.z; r1.w += c * v1.w;
        *reinterpret_cast<float4*>(row + j0) = r0;
        if (two) *reinterpret_cast<float4*>(row + j0 + 4) = r1;
    }
}

// lane i < K: sum_j P[i][j] v[j] (v in LDS, zero beyond K); other lanes 0
__device__ __forceinline__ float inv_matvec(const float* P, int K, const float* v, int lane) {
    const float* row = P + (lane < K ? lane : 0) * IN_PS;
    float a0 = 0.f, a1 = 0.f;
    for (int j0 = 0; j0 < K; j0 += 8) {
        const float4 r0 = *reinterpret_cast<const float4*>(row + j0), v0 = *reinterpret_cast<const float4*>(v + j0);
        a0 += r0.x * v0.x + r0.y * v0.y + r0.z * v0.z + r0.w * v0.w;
        if (j0 + 4 < K) {                                // uniform
            const float4 r1 = *reinterpret_cast<const float4*>(row + j0 + 4), v1 = *reinterpret_cast<const float4*>(v + j0 + 4);
            a1 += r1.x * v1.x + r1.y * v1.y + r1.z * v1.z + r1.w * v1.w;
        }
    }
    return lane < K ? a0 + a1 : 0.f;
}

// Unit u enters at position K (K < 64).  tmp: 2 * 64 floats of LDS.  Returns 1 when the Schur complement is
// not positive (u depends linearly on the list, or repeats one of its units).
__device__ __forceinline__ int inv_append(const float* gram, int N, int* S, int K, int u, float* P, float* tmp, int lane) {
    float* gS = tmp;
    float* wv = tmp + SD_MAXK;
    const float g = lane < K ? gram[(size_t)u * N + S[lane]] : 0.f;
    gS[lane] = g;
    inc_wave_fence();
    const float w = inv_matvec(P, K, gS, lane);
    const float sc = gram[(size_t)u * N + u] - wave_sum(g * w);
    const bool ok = sc > 0.f;
    const float is = ok ? 1.0f / sc : 0.f;
    wv[lane] = w;                                         // zero beyond K
    inc_wave_fence();
    if (lane < K) {
        float* row = P + lane * IN_PS;
        const float wi = w * is;
        inv_row_axpy(row, K, wi, wv);
        row[K] = -wi;
        P[K * IN_PS + lane] = -wi;
    }
    if (lane == 0) { P[K * IN_PS + K] = is; S[K] = u; }
    inc_wave_fence();
    return ok ? 0 : 1;
}

// The unit at position j leaves a list of K units; the last unit of the list takes its place.
__device__ __forceinline__ void inv_remove(int* S, int K, int j, float* P, float* tmp, int lane) {
    float* cv = tmp;
    const float col = lane < K ? P[lane * IN_PS + j] : 0.f;
    const float dj = P[j * IN_PS + j];
    const float id = dj > 0.f ? 1.0f / dj : 0.f;
    cv[lane] = col;                                       // zero beyond K
    inc_wave_fence();
    if (lane < K && lane != j) inv_row_axpy(P + lane * IN_PS, K, -col * id, cv);
    inc_wave_fence();
    const int last = K - 1;
    // row and column `last` move to j (entries (., j) and (j, .) of the unit that left are dead), and the
    // place they leave is cleared
    const float lastcol = lane < last ? P[lane * IN_PS + last] : 0.f;          // = P[last][lane]: symmetric
    const float corner = P[last * IN_PS + last];
    inc_wave_fence();
    if (lane < K) { P[lane * IN_PS + last] = 0.f; P[last * IN_PS + lane] = 0.f; }
    inc_wave_fence();
    if (j != last) {
        if (lane < last && lane != j) { P[lane * IN_PS + j] = lastcol; P[j * IN_PS + lane] = lastcol; }
        if (lane == j) P[j * IN_PS + j] = corner;
        if (lane == 0) S[j] = S[last];
    }
    inc_wave_fence();
}

template <bool GRAM_LDS>
__global__ __launch_bounds__(IN_THREADS)
void recover_carry_kernel(Plan p, RecoverArgs a, IncArgs q, IncLayout L) {
    extern __shared__ __attribute__((aligned(16))) float lds_carry[];
    float* lds = lds_carry;
    const int tid = threadIdx.x, NT = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nwaves = NT >> 6;
    const int prob = blockIdx.x;
    const int N = p.N, m = p.op.m, k = a.k;
    const int swaps = q.swaps, K0 = k - swaps;
    const bool active = tid < N;

    float* yv = lds + L.off_y;
    float* rv = lds + L.off_r;
    float* c0v = lds + L.off_c0;
    float* nrm = lds + L.off_nrm;
    int* flag = reinterpret_cast<int*>(lds + L.off_flag);
    int* S = reinterpret_cast<int*>(lds + L.off_S);
    float* c0S = lds + L.off_S2;                // c0 of the listed units, in list order
    float* tv = lds + L.off_t;                  // [4][IN_MAXK] small vectors
    float* P = lds + L.off_L;                   // inverse of G_SS, row stride IN_PS
    int* misc = reinterpret_cast<int*>(lds + L.off_misc);
    float* red = lds + L.off_red;
    float* stage = lds + L.off_stage;
    float* gram_l = lds + L.off_gram;
    const float* gram = GRAM_LDS ? gram_l : p.gram;
    float* xs = tv, *tmp = tv + IN_MAXK, *dl = tv + 3 * IN_MAXK;     // tmp: two vectors

    uint32_t* state = q.state + (size_t)prob * q.state_stride;
    const float* y = a.y + (size_t)prob * m;
    int bad = 0;
    float iw = 1.f, w = 1.f;                           // W holds 1/norm of the atom
    if (active && p.weighted) { iw = p.W[tid]; w = iw > 0.f ? 1.0f / iw : 0.f; }
    if (active) { nrm[tid] = w; flag[tid] = 0; }
    for (int e = tid; e < IN_MAXK * IN_PS; e += NT) P[e] = 0.f;
    // previous support: in range and without repeats, else the row is reported as failed
    if (wave == 0) {
        const int u = lane < k ? q.prev_support[(size_t)prob * k + lane] : -1;
        int ok = lane >= k || (u >= 0 && u < p.G);
        for (int i = 0; i < k; ++i) {
            const int ui = __builtin_amdgcn_readlane(u, i);
            if (lane < k && lane != i && ui == u) ok = 0;
        }
        if (!ok) bad = 1;
        S[lane] = (lane < k && ok) ? u : 0;
        xs[lane] = 0.f;
    }
    // the state's header and list are requested with the other start-up loads
    const uint32_t hdr = state[0], age = state[1];
    const int su_state = tid < k ? (int)state[2 + tid] : 0;
    const float c0 = load_sketch_gram_c0<GRAM_LDS>(p, y, yv, gram_l, stage, bad);
    if (active) c0v[tid] = c0;
    if (tid == 0) misc[0] = 0;
    __syncthreads();
    if (bad) {                                           // uniform: NaN sketch or invalid previous support
        for (int i = tid; i < k; i += NT) {
            a.support[(size_t)prob * k + i] = -1;
            if (a.coef) a.coef[(size_t)prob * k + i] = 0.f;
        }
        if (tid == 0) {
            if (a.resid) a.resid[prob] = __int_as_float(0x7fc00000);
            if (a.margin) a.margin[prob] = 0.f;
            state[0] = 0u;
        }
        return;
    }
    // ---- the state is used when it was left for exactly this set of units and is not too old
    if (tid < k) flag[S[tid]] = 2;
    __syncthreads();
    int usable = hdr == (IN_MAGIC | (uint32_t)k) && age < (uint32_t)IN_REFRESH;
    if (tid < k && !(su_state >= 0 && su_state < p.G && flag[su_state < p.G && su_state >= 0 ? su_state : 0] == 2)) usable = 0;
    usable = !__syncthreads_or(!usable);                 // also orders the reads of flag[] before it is cleared
    if (tid < k) flag[S[tid]] = 0;
    if (usable) {
        if (tid < k) S[tid] = su_state;                  // k distinct units of the set: the same set in the state's order
        const float* ps = reinterpret_cast<const float*>(state + 2 + k);
        for (int e = tid; e < k * k; e += NT) P[(e / k) * IN_PS + (e % k)] = ps[e];
    }
    __syncthreads();

    // ---- 1./2. fit on the previous support, backward step (wavefront 0)
    if (wave == 0) {
        int wbad = 0;
        if (!usable && swaps < k)
            for (int i = 0; i < k; ++i) wbad |= inv_append(gram, N, S, i, S[i], P, tmp, lane);
        int K = swaps < k ? k : 0;
        if (K > 0) {
            const int su = lane < k ? S[lane] : 0;
            c0S[lane] = lane < k ? c0v[su] : 0.f;
            inc_wave_fence();
            const float x = inv_matvec(P, k, c0S, lane);
            if (swaps == 0) {
                xs[lane] = x;
            } else {
                // the `swaps` weakest units leave (rank 0 = strongest; equal energies: smaller index first)
                float e = lane < k ? x * nrm[su] : -1.f;
                e = e * e;
                if (lane >= k) e = -1.f; else if (!(e >= 0.f)) e = 0.f;
                int rank = 0;
                for (int i = 0; i < k; ++i) {
                    const float ei = readlane_f32(e, i);
                    const int ui = __builtin_amdgcn_readlane(su, i);
                    rank += (int)(ei > e) | ((int)(ei == e) & (int)(ui < su));
                }
                unsigned long long leave = __ballot(lane < k && rank >= K0);
                while (leave) {                          // from the back: the unit that fills a gap is one that stays
                    const int j = 63 - __builtin_clzll(leave);
                    leave &= ~(1ull << j);
                    inv_remove(S, K, j, P, tmp, lane);
                    --K;
                }
                c0S[lane] = lane < K ? c0v[S[lane]] : 0.f;
                inc_wave_fence();
                xs[lane] = inv_matvec(P, K, c0S, lane);
            }
        }
        if (lane == 0) misc[0] = wbad;
        inc_wave_fence();
    }
    __syncthreads();
    if (tid < K0) flag[S[tid]] = 1;
    __syncthreads();

    // ---- 3. forward step
    float margin = 1.f;
    unsigned long long* redk = reinterpret_cast<unsigned long long*>(red);       // [nwaves] best keys
    float* red2 = red + 32;                                                       // [nwaves] runner-up scores
    for (int it = 0; it < swaps; ++it) {
        const int K = K0 + it;
        // correlation with the residual of the current fit: c0 - G[:, S] alpha.  The list and its coefficients
        // are read four at a time from LDS (every lane the same address); entries K .. of the list are
        // units that have left or zero, with coefficient zero.
        const int ta = active ? tid : 0;
        float acc = 0.f;
        for (int j = 0; j < K; j += 4) {
            const int4 s4 = *reinterpret_cast<const int4*>(S + j);
            const float4 a4 = *reinterpret_cast<const float4*>(xs + j);
            acc += a4.x * gram[(size_t)s4.x * N + ta] + a4.y * gram[(size_t)s4.y * N + ta] +
                   a4.z * gram[(size_t)s4.z * N + ta] + a4.w * gram[(size_t)s4.w * N + ta];
        }
        float sc = iw * (c0 - acc);
        sc = sc * sc;
        if (!(sc >= 0.f)) sc = 0.f;
        const bool cand = active && flag[tid] == 0;
        unsigned long long key = cand ? ((unsigned long long)__float_as_uint(sc) << 32) | (0xffffffffu - (unsigned)tid) : 0ull;
        unsigned long long kb = key;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long o = __shfl_xor(kb, off);
            kb = o > kb ? o : kb;
        }
        const float s2w = wave_max(cand && key != kb ? sc : -1.f);
        if (lane == 0) { redk[wave] = kb; red2[wave] = s2w; }
        __syncthreads();
        unsigned long long gb = 0ull;
        for (int wv = 0; wv < nwaves; ++wv) { const unsigned long long o = redk[wv]; gb = o > gb ? o : gb; }
        float s2 = 0.f;
        for (int wv = 0; wv < nwaves; ++wv) {
            const unsigned long long o = redk[wv];
            if (o != gb && o != 0ull) s2 = fmaxf(s2, __uint_as_float((unsigned)(o >> 32)));
            s2 = fmaxf(s2, red2[wv]);
        }
        const float s1 = __uint_as_float((unsigned)(gb >> 32));
        const int best = min(max((int)(0xffffffffu - (unsigned)(gb & 0xffffffffull)), 0), N - 1);   // always a candidate: K < k <= N
        margin = fminf(margin, s1 > 0.f ? (s1 - s2) / s1 : 0.f);
        if (wave == 0) {
            const int wbad = inv_append(gram, N, S, K, best, P, tmp, lane);
            if (lane == 0) { flag[best] = 1; if (wbad) misc[0] = 1; }
            c0S[lane] = lane <= K ? c0v[S[lane]] : 0.f;
            inc_wave_fence();
            xs[lane] = inv_matvec(P, K + 1, c0S, lane);
            inc_wave_fence();
        }
        __syncthreads();
    }
    bad = misc[0];

    // ---- 4. explicit residual and one refinement step on the final support
    const bool want_fit = a.coef != nullptr || a.resid != nullptr;
    float* gvv = tmp;                                     // M_S^T r
    float* part = tmp + IN_MAXK;                          // per-wave partial sums
    if (want_fit) {
        for (int i = tid; i < m; i += NT) {
            float s = yv[i];
            for (int j = 0; j < k; ++j) s -= xs[j] * p.Mr[(size_t)i * N + S[j]];
            rv[i] = s;
        }
        __syncthreads();
        for (int j = wave; j < k; j += nwaves) {
            float s = 0.f;
            for (int i = lane; i < m; i += 64) s += p.Mr[(size_t)i * N + S[j]] * rv[i];
            s = wave_sum(s);
            if (lane == 0) gvv[j] = s;
        }
        if (tid >= k && tid < IN_MAXK) gvv[tid] = 0.f;   // the product below runs to the next multiple of four
        __syncthreads();
        if (wave == 0) {
            const float d = inv_matvec(P, k, gvv, lane);
            if (lane < k) { xs[lane] += d; dl[lane] = d; }
        }
        __syncthreads();
        float ss = 0.f;
        for (int i = tid; i < m; i += NT) {
            float s = rv[i];
            for (int j = 0; j < k; ++j) s -= dl[j] * p.Mr[(size_t)i * N + S[j]];
            ss += s * s;
        }
        ss = wave_sum(ss);
        if (lane == 0) part[wave] = ss;
        __syncthreads();
    }
    for (int qi = tid; qi < k; qi += NT) {
        const int gsel = S[qi];
        int rank = 0;
        for (int o = 0; o < k; ++o) rank += S[o] < gsel;
        a.support[(size_t)prob * k + rank] = gsel;
        if (a.coef) a.coef[(size_t)prob * k + rank] = xs[qi];
    }
    // ---- what the next token starts from
    if (!bad) {
        float* ps = reinterpret_cast<float*>(state + 2 + k);
        for (int e = tid; e < k * k; e += NT) ps[e] = P[(e / k) * IN_PS + (e % k)];
        if (tid < k) state[2 + tid] = (uint32_t)S[tid];
    }
    if (tid == 0) {
        state[0] = bad ? 0u : (IN_MAGIC | (uint32_t)k);
        state[1] = usable ? age + 1u : 1u;
        if (a.resid) {
            float tot = 0.f;
            for (int wv = 0; wv < nwaves; ++wv) tot += part[wv];
            a.resid[prob] = bad ? __int_as_float(0x7fc00000) : sqrtf(tot);
        }
        if (a.margin) a.margin[prob] = bad ? 0.f : margin;
    }
}

size_t recover_inc_state_words(int k) { return (size_t)((2 + k + k * k + 3) & ~3); }

hipError_t launch_recover_carry(const Plan& p, const RecoverArgs& a, const IncArgs& q, int lds_limit, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    IncLayout L;
    // without an exchange the Gram matrix is not read at all: no copy of it in LDS
    if (!make_inc_layout(p, lds_limit, IN_THREADS, L, q.swaps > 0)) return hipErrorInvalidValue;
    const size_t bytes = (size_t)L.total_floats * 4;
    if (L.off_gram >= 0) {
        static size_t allowed = 0;
        if (bytes > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_carry_kernel<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            allowed = bytes;
        }
        hipLaunchKernelGGL(recover_carry_kernel<true>, dim3(a.B), dim3(IN_THREADS), bytes, s, p, a, q, L);
    } else {
        static size_t allowed = 0;
        if (bytes > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_carry_kernel<false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            allowed = bytes;
        }
        hipLaunchKernelGGL(recover_carry_kernel<false>, dim3(a.B), dim3(IN_THREADS), bytes, s, p, a, q, L);
    }
    return hipGetLastError();
}

bool recover_inc_supported(const Plan& p, int k, int lds_limit) {
    if (p.rb != 1 || k > IN_MAXK || p.N > IN_THREADS) return false;
    IncLayout L;
    const int nthreads = (p.N <= 64 && p.op.m <= 64) ? 64 : IN_THREADS;
    return make_inc_layout(p, lds_limit, nthreads, L);
}

hipError_t launch_recover_inc(const Plan& p, const RecoverArgs& a, const IncArgs& q, int lds_limit, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    const int nthreads = (p.N <= 64 && p.op.m <= 64) ? 64 : IN_THREADS;
    IncLayout L;
    if (!make_inc_layout(p, lds_limit, nthreads, L)) return hipErrorInvalidValue;
    const size_t bytes = (size_t)L.total_floats * 4;
    if (L.off_gram >= 0) {
        static size_t allowed = 0;
        if (bytes > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_inc_kernel<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            allowed = bytes;
        }
        hipLaunchKernelGGL(recover_inc_kernel<true>, dim3(a.B), dim3(nthreads), bytes, s, p, a, q, L);
    } else {
        static size_t allowed = 0;
        if (bytes > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(recover_inc_kernel<false>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            allowed = bytes;
        }
        hipLaunchKernelGGL(recover_inc_kernel<false>, dim3(a.B), dim3(nthreads), bytes, s, p, a, q, L);
    }
    return hipGetLastError();
}

}  // namespace csk
