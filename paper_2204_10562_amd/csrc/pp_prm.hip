// Partition, replication and mapping (PRM, Alg. 4; recursion for W(l, xi, r, i) in Sec. IV-B)
// for a batch of device orderings: the dynamic program over (layers, stages, replicas of the
// last stage, GPUs used) with the AllReduce term of Eq. 1, for every stage count at once.
//
//   W(l, xi, r, i) = min over l' in [xi-1, l-1], r' in [1, i-r] of
//                    max{ W(l', xi-1, r', i-r),  M (c^f + c^b),  M (F + B) + A }
//   W(l, 1, i, i)  = M (F + B) + A of layers [0, l) on all i GPUs
// where, for the last stage = layers [l', l) on the r GPUs of ranks [i-r, i):
//   F = ceil(sum p^f / r), B = ceil(sum p^b / r)            (per-replica times, Sec. III-B)
//   A = ceil(2 (r-1) sum alpha / (r min b)), 0 for r = 1    (Eq. 1; min over the replica set)
//   c^f = ceil(d^f / (r' r min b_{v',v})), c^b = ceil(d^b / (r' r min b_{v,v'}))
//         (v' in the r' GPUs of ranks [i-r-r', i-r), v in the last stage's).
// The listing scans l' ascending, then r' ascending, and replaces its best only on strict
// improvement: the minimiser kept is the first in (l', r') order.
//
// One workgroup per candidate (persistent over candidates), one thread per cell l.  State
// (xi, r, i) depends only on states with fewer GPUs, so states are visited by ascending i.
// All states with the same (r, i) share the last stage's terms, which are made division-free:
// with Q[l] = floor(P[l] / r), R[l] = P[l] mod r,  ceil((P[l] - P[l']) / r) =
// Q[l] - Q[l'] + (R[l] > R[l']); so the stage term is U[l] - U[l'] + (remainder compares) with
// U = M (QF + QB) + QA; the channel term X[r'][l'] = M (c^f + c^b) is computed once per (r, i)
// too.  Neither the sub-problem nor the channel term depends on l, and the last stage's term
// does not depend on r'; max with the latter commutes with the minimum over r', so per state
//   Gmin[l'] = min over r' of max(W(l', xi-1, r', i-r), X[r'][l'])
// is built once in LDS and a cell costs one pass over l' only:
//   W(l, xi, r, i) = min over l' of max(Gmin[l'], last stage [l', l)).
// The r' that goes with the chosen l' is then the first one whose value reaches the minimum.
// States that use all D GPUs are needed at l = L only and are reduced by the whole workgroup.
#include "pp_common.h"

#define PRM_THREADS 128

struct prm_args {
    int L, D, M;
    long long N;
    const long long *fwd, *bwd, *actf, *actb, *alpha, *bw;
    const int *ord;  // [N][D]
    char *scratch;   // slots * slot_bytes
    size_t slot_bytes;
    long long *W_out;  // [N][D]: W of the best plan with xi stages at xi-1 (PP_INF64: none)
    int *bounds_out;   // [N][D(D+1)/2]
    int *reps_out;     // [N][D(D+1)/2]
    long long *pre_out;  // [3][L+1]: prefix sums of fwd, bwd, alpha for the kernels that follow
    int32_t *status;
};

__host__ __device__ static inline int prm_states(int D) { return D * (D + 1) * (D + 2) / 6; }

// Index of state (i GPUs, xi stages, r replicas of the last stage), 1 <= xi <= i,
// 1 <= r <= i - xi + 1.
__host__ __device__ static inline int prm_sid(int i, int xi, int r) {
    return (i - 1) * i * (i + 1) / 6 + (xi - 1) * (i + 1) - xi * (xi - 1) / 2 + (r - 1);
}

// Bytes of per-workgroup scratch: W and the minimising (l', r') of every state and cell, and
// the minima of the bandwidth matrix over rank sets.
static inline size_t prm_slot_bytes(int L, int D) {
    size_t cells = (size_t)prm_states(D) * (L + 1);
    size_t minima = (size_t)(D + 1) * (D + 1) * (D + 1) * 2 + (size_t)(D + 1) * (D + 1);
    return pp_align256(cells * 8) + pp_align256(cells * 4) + pp_align256(minima * 8);
}

static inline size_t prm_lds_bytes(int L, int D) {
    // PF, PB, PA (int64), one row record per layer position (32 bytes in the int64 form),
    // X (int64, D-1 rows)
    // (the three prefix arrays are padded to an even length so that the records are 16-byte aligned)
    return (size_t)(L + 2) * (3 * 8) + (size_t)(L + 1) * 32 + (size_t)(D > 1 ? D - 1 : 1) * (L + 1) * 8 + 64;
}

struct prm_key {
    long long v;
    int lp, rp;
};

__device__ __forceinline__ bool prm_less(const prm_key &a, const prm_key &b) {
    if (a.v != b.v) return a.v < b.v;
    if (a.lp != b.lp) return a.lp < b.lp;
    return a.rp < b.rp;
}

__device__ __forceinline__ long long cdiv64(long long a, long long b) { return a / b + (a % b != 0); }

// Values are int64, or int32 when every finite value of the launch is known to stay below
// 2^30 (decided on the device from bounds on the stage and channel terms).
template <bool WIDE> struct prm_val { using V = int; };
template <> struct prm_val<true> { using V = long long; };

// What the cell loop reads per layer position l' (one LDS access in the int32 form):
//   g  = Gmin[l'] of the current state
//   u  = U[l'], ra = remainder of the AllReduce quotient   (current (r, i))
//   oh = (1 << RF[l']) | (1 << (16 + RB[l'])), the remainders of the two compute quotients as
//        one-hot bits, so that [RF[l] > RF[l']] + [RB[l] > RB[l']] is the popcount of oh
//        masked with ((1 << RF[l]) - 1) | (((1 << RB[l]) - 1) << 16).
template <bool WIDE> struct alignas(16) prm_row { int g, u, ra, oh; };
template <> struct alignas(16) prm_row<true> { long long g, u, ra; int oh, pad; };

struct prm_shared {
    int o[PP_MAX_STAGES];
    int fault, keep, wide;
    unsigned long long amax_f, amax_b, bmin, bmax;
    prm_key red[PRM_THREADS / 64];
};

template <bool WIDE>
__device__ void prm_run(const prm_args &a, unsigned char *smem, prm_shared &sh) {
    using V = typename prm_val<WIDE>::V;
    using Row = prm_row<WIDE>;
    const V INF = WIDE ? (V)PP_INF64 : (V)PP_INF32;
    const int L = a.L, D = a.D, tid = threadIdx.x, B = blockDim.x;
    const long long M = a.M;
    const V Mv = (V)a.M;
    const int L1 = L + 1, D1 = D + 1;
    const int L1p = (L1 + 1) & ~1;  // even, so that what follows the int64 arrays is 16-byte aligned
    long long *PF = (long long *)smem, *PB = PF + L1p, *PA = PB + L1p;
    Row *Q = (Row *)(PA + L1p);                          // [L1]
    V *X = (V *)((long long *)(PA + L1p) + 4 * (size_t)L1);  // [D-1][L1], after 32 bytes per record
    const int NS = prm_states(D), tri = D * (D + 1) / 2;
    char *slot = a.scratch + (size_t)blockIdx.x * a.slot_bytes;
    V *Wt = (V *)slot;                                                   // [NS][L1]
    unsigned *At = (unsigned *)(slot + pp_align256((size_t)NS * L1 * 8));  // l' | r' << 16
    long long *bfwd = (long long *)((char *)At + pp_align256((size_t)NS * L1 * 4));  // [p][rp][r]
    long long *bbwd = bfwd + (size_t)D1 * D1 * D1;
    long long *bin = bbwd + (size_t)D1 * D1 * D1;                        // [n][r]

    // A workgroup walks a contiguous chunk of candidates.  State (xi, r, i) depends only on the
    // first i devices of the ordering, so whatever the previous candidate shares as a prefix is
    // kept (with all D! orderings in lexicographic order most of the table is).
    const long long chunk = (a.N + gridDim.x - 1) / gridDim.x;
    const long long c_first = (long long)blockIdx.x * chunk;
    const long long c_end = c_first + chunk < a.N ? c_first + chunk : a.N;
    bool have_prev = false;
    for (long long c = c_first; c < c_end; ++c) {
        __syncthreads();
        // ---- ordering
        if (tid == 0) {
            int bad = 0, same = 0;
            bool eq = have_prev;
            for (int n = 0; n < D; ++n) {
                int d = a.ord[c * D + n];
                if (d < 0 || d >= D) bad = 1;
                for (int q = 0; q < n; ++q) bad |= (sh.o[q] == d);
                eq = eq && sh.o[n] == d;
                same += eq;
                sh.o[n] = d;
            }
            sh.fault = bad;
            sh.keep = same < D ? same : D - 1;  // the states on all D GPUs are always redone
        }
        __syncthreads();
        const int keep = sh.keep;
        have_prev = !sh.fault;
        if (sh.fault) {
            if (tid == 0) pp_raise(a.status, PP_FAULT_ORDERING);
            for (int n = tid; n < D; n += B) a.W_out[c * D + n] = PP_INF64;
            for (int n = tid; n < tri; n += B) { a.bounds_out[c * tri + n] = 0; a.reps_out[c * tri + n] = 0; }
            continue;
        }
        const int *o = sh.o;
        // ---- minima of the bandwidth matrix over rank sets
        // bfwd[p][rp][r]: links from ranks [p-rp, p) to ranks [p, p+r); bbwd: the other direction
        for (int t = tid; t < D1 * D1 * D1; t += B) {
            const int p = t / (D1 * D1), rp = (t / D1) % D1, r = t % D1;
            if (p < 1 || rp < 1 || r < 1 || rp > p || p + r > D || p + r <= keep) continue;
            long long mf = PP_INF64, mb = PP_INF64;
            for (int u = p - rp; u < p; ++u)
                for (int v = p; v < p + r; ++v) {
                    long long x = a.bw[(size_t)o[u] * D + o[v]], y = a.bw[(size_t)o[v] * D + o[u]];
                    mf = x < mf ? x : mf;
                    mb = y < mb ? y : mb;
                }
            bfwd[t] = mf;
            bbwd[t] = mb;
        }
        // bin[n][r]: ordered pairs inside ranks [n-r, n)
        for (int t = tid; t < D1 * D1; t += B) {
            const int n = t / D1, r = t % D1;
            if (n < 1 || r < 2 || r > n || n <= keep) continue;
            long long m = PP_INF64;
            for (int u = n - r; u < n; ++u)
                for (int v = n - r; v < n; ++v)
                    if (u != v) {
                        long long x = a.bw[(size_t)o[u] * D + o[v]];
                        m = x < m ? x : m;
                    }
            bin[t] = m;
        }
        __syncthreads();

        // ---- states by ascending number of GPUs
        for (int i = keep + 1; i <= D; ++i) {
            const bool top = i == D;  // all GPUs in use: only cell L is needed
            for (int r = 1; r <= i; ++r) {
                // Last stage on r replicas, ranks [i-r, i): division-free form of its terms, and
                // the channel term X[r'][l'] = M (c^f + c^b) towards r' replicas on ranks
                // [i-r-r', i-r); both are shared by every stage count.
                const long long den = r > 1 ? (long long)r * bin[i * D1 + r] : 1;
                for (int l = tid; l <= L; l += B) {
                    long long qf = PF[l] / r, qb = PB[l] / r;
                    long long num = 2 * (long long)(r - 1) * PA[l];
                    long long qa = num / den;
                    Q[l].u = (V)(M * (qf + qb) + qa);
                    Q[l].ra = (V)(num - qa * den);
                    Q[l].oh = (1 << (int)(PF[l] - qf * r)) | (1 << (16 + (int)(PB[l] - qb * r)));
                }
                const int n0 = i - r;  // GPUs of the sub-problem
                for (int t = tid; t < n0 * L1; t += B) {
                    const int rp = 1 + t / L1, lp = t % L1;
                    V x = INF;
                    if (lp >= 1 && lp <= L - 1) {
                        const size_t at = ((size_t)n0 * D1 + rp) * D1 + r;
                        x = (V)(M * (cdiv64(a.actf[lp - 1], (long long)rp * r * bfwd[at]) +
                                     cdiv64(a.actb[lp - 1], (long long)rp * r * bbwd[at])));
                    }
                    X[(size_t)(rp - 1) * L1 + lp] = x;
                }
                __syncthreads();
                // the last stage [l', l): M (F + B) + A, from the records of l' and l
                auto last_stage = [&](const Row &q, const Row &ql, int mask) -> V {
                    const int flags = __popc((unsigned)(q.oh & mask));  // 0, 1 or 2
                    const V extra = WIDE ? Mv * (V)flags : (V)__mul24(flags, (int)Mv);  // M < 2^20 here
                    return ql.u - q.u + extra + (V)(ql.ra > q.ra);
                };
                auto mask_of = [](int oh) -> int {
                    // remainders (f, b) one-hot at bits f and 16 + b -> all lower bits of each half
                    return oh - 0x10001;
                };
                for (int xi = 1; xi <= i - r + 1; ++xi) {
                    const int sid = prm_sid(i, xi, r);
                    V *Ws = Wt + (size_t)sid * L1;
                    unsigned *As = At + (size_t)sid * L1;
                    if (xi == 1) {
                        // a single stage must take all i GPUs
                        for (int l = top ? L + tid : tid; l <= L; l += B) {
                            Ws[l] = (r == i && l >= 1) ? last_stage(Q[0], Q[l], mask_of(Q[l].oh)) : INF;
                            As[l] = 0;
                        }
                        continue;  // touches no LDS array that the next state rewrites
                    }
                    const int nrp = n0 - (xi - 2);  // r' = 1..nrp leave >= 1 GPU per earlier stage
                    // Gmin[l'] = min over r' of max(W(l', xi-1, r', n0), X[r'][l']).  The last
                    // stage's term does not depend on r', and max with it commutes with this min.
                    for (int lp = tid; lp <= L; lp += B) {
                        V g = INF;
                        if (lp >= xi - 1 && lp <= L - 1) {
                            // four loads in flight at a time; a clamped r' repeats the last one
                            const V *Wsub = Wt + (size_t)prm_sid(n0, xi - 1, 1) * L1 + lp;  // r' = 1, 2, ...
                            for (int rp0 = 1; rp0 <= nrp; rp0 += 4) {
                                V w[4], x[4];
#pragma unroll
                                for (int k = 0; k < 4; ++k) {
                                    const int rp = rp0 + k <= nrp ? rp0 + k : nrp;
                                    w[k] = Wsub[(size_t)(rp - 1) * L1];
                                    x[k] = X[(size_t)(rp - 1) * L1 + lp];
                                }
#pragma unroll
                                for (int k = 0; k < 4; ++k) {
                                    const V m = w[k] > x[k] ? w[k] : x[k];
                                    g = m < g ? m : g;
                                }
                            }
                        }
                        Q[lp].g = g;
                    }
                    __syncthreads();
                    // first r' (ascending) whose value reaches the minimum v found at l'
                    auto first_rp = [&](int lp, int l, V v) -> int {
                        const V last = last_stage(Q[lp], Q[l], mask_of(Q[l].oh));
                        for (int rp = 1; rp <= nrp; ++rp) {
                            V w = Wt[(size_t)prm_sid(n0, xi - 1, rp) * L1 + lp];
                            V x = X[(size_t)(rp - 1) * L1 + lp];
                            w = w > x ? w : x;
                            if ((w > last ? w : last) == v) return rp;
                        }
                        return 0;
                    };
                    if (!top) {
                        for (int l = tid; l <= L; l += B) {
                            const Row ql = Q[l];
                            const int mask = mask_of(ql.oh);
                            V best = INF;
                            int blp = 0;
                            // Splits from l-1 downwards: the last stage's term grows as l'
                            // falls, so once it alone exceeds the best value no lower l' can
                            // match it.  '<=' keeps the lowest l' among equal values, which is
                            // what the ascending scan with '<' of the listing keeps.
                            int lp = l - 1;
                            for (; lp - 3 >= xi - 1; lp -= 4) {
                                Row q[4];
#pragma unroll
                                for (int k = 0; k < 4; ++k) q[k] = Q[lp - k];
                                V last = 0;
#pragma unroll
                                for (int k = 0; k < 4; ++k) {
                                    last = last_stage(q[k], ql, mask);
                                    const V t = q[k].g > last ? q[k].g : last;
                                    if (t <= best) { best = t; blp = lp - k; }
                                }
                                if (last > best) { lp = xi - 2; break; }  // nothing below can win
                            }
                            for (; lp >= xi - 1; --lp) {
                                const Row q = Q[lp];
                                const V last = last_stage(q, ql, mask);
                                if (last > best) break;
                                const V t = q.g > last ? q.g : last;
                                if (t <= best) { best = t; blp = lp; }
                            }
                            Ws[l] = best;
                            As[l] = best == INF ? 0u : ((unsigned)blp | ((unsigned)first_rp(blp, l, best) << 16));
                        }
                    } else {
                        // the workgroup shares the scan of l' for the single cell L
                        const Row ql = Q[L];
                        const int mask = mask_of(ql.oh);
                        prm_key best = {PP_INF64, 0, 0};
                        for (int lp = xi - 1 + tid; lp < L; lp += B) {
                            const Row q = Q[lp];
                            const V last = last_stage(q, ql, mask);
                            const V t = q.g > last ? q.g : last;
                            prm_key k = {t == INF ? PP_INF64 : (long long)t, lp, 0};
                            if (prm_less(k, best)) best = k;
                        }
                        for (int off = 32; off; off >>= 1) {
                            prm_key ok;
                            ok.v = __shfl_xor(best.v, off);
                            ok.lp = __shfl_xor(best.lp, off);
                            ok.rp = 0;
                            if (prm_less(ok, best)) best = ok;
                        }
                        if ((tid & 63) == 0) sh.red[tid >> 6] = best;
                        __syncthreads();
                        if (tid == 0) {
                            for (int w = 1; w < B / 64; ++w)
                                if (prm_less(sh.red[w], best)) best = sh.red[w];
                            const bool none = best.v == PP_INF64;
                            Ws[L] = none ? INF : (V)best.v;
                            As[L] = none ? 0u : ((unsigned)best.lp | ((unsigned)first_rp(best.lp, L, (V)best.v) << 16));
                        }
                    }
                    __syncthreads();  // the g fields (and sh.red) are rewritten by the next state
                }
                __syncthreads();  // the records and X are rewritten by the next (r, i)
            }
        }

        // ---- per stage count: the first r with the smallest W (Alg. 3), and its plan
        __threadfence_block();
        __syncthreads();
        for (int xi = 1 + tid; xi <= D; xi += B) {
            V wbest = INF;
            int rbest = 0;
            for (int r = 1; r <= D - xi + 1; ++r) {
                V w = Wt[(size_t)prm_sid(D, xi, r) * L1 + L];
                if (w < wbest) { wbest = w; rbest = r; }
            }
            a.W_out[c * D + xi - 1] = wbest == INF ? PP_INF64 : (long long)wbest;
            int *bo = a.bounds_out + c * tri + xi * (xi - 1) / 2;
            int *ro = a.reps_out + c * tri + xi * (xi - 1) / 2;
            int l = L, n = D, r = rbest;
            for (int s = xi - 1; s >= 0; --s) {
                if (wbest == INF) { bo[s] = 0; ro[s] = 0; continue; }
                bo[s] = l;
                ro[s] = r;
                unsigned arg = At[(size_t)prm_sid(n, s + 1, r) * L1 + l];
                n -= r;
                l = (int)(arg & 0xffffu);
                r = (int)(arg >> 16);
            }
        }
    }
}

__global__ __launch_bounds__(PRM_THREADS) void k_prm(prm_args a) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ prm_shared sh;
    const int L = a.L, D = a.D, tid = threadIdx.x, B = blockDim.x;
    const long long M = a.M;
    const int L1 = L + 1, L1p = (L1 + 1) & ~1;
    long long *PF = (long long *)smem, *PB = PF + L1p, *PA = PB + L1p;

    // prefix sums (every workgroup makes its own copy: L is small next to the DP), input checks
    // and the bounds that decide between int32 and int64 values
    if (tid == 0) {
        sh.fault = 0;
        sh.amax_f = sh.amax_b = sh.bmax = 0;
        sh.bmin = ~0ull;
    }
    __syncthreads();
    {
        int fault = 0;
        unsigned long long af = 0, ab = 0, lo = ~0ull, hi = 0;
        for (int l = tid; l < L; l += B) {
            long long x = a.fwd[l], y = a.bwd[l], z = a.alpha[l];
            if (x < 0 || y < 0 || z < 0) fault |= PP_FAULT_NEGATIVE;
            if (l + 1 < L) {
                long long f = a.actf[l], b = a.actb[l];
                if (f < 0 || b < 0) fault |= PP_FAULT_NEGATIVE;
                af = (unsigned long long)f > af ? (unsigned long long)f : af;
                ab = (unsigned long long)b > ab ? (unsigned long long)b : ab;
            }
            if (x >= PP_CAP62 || y >= PP_CAP62 || z >= PP_CAP62) fault |= PP_FAULT_OVERFLOW;
            PF[l + 1] = x; PB[l + 1] = y; PA[l + 1] = z;
        }
        for (int t = tid; t < D * D; t += B)
            if (t / D != t % D) {
                long long b = a.bw[t];
                if (b <= 0) fault |= PP_FAULT_BANDWIDTH;
                lo = (unsigned long long)b < lo ? (unsigned long long)b : lo;
                hi = (unsigned long long)b > hi ? (unsigned long long)b : hi;
            }
        if (fault) atomicOr(&sh.fault, fault);
        atomicMax(&sh.amax_f, af);
        atomicMax(&sh.amax_b, ab);
        atomicMax(&sh.bmax, hi);
        atomicMin(&sh.bmin, lo);
    }
    __syncthreads();
    if (tid == 0 && !sh.fault) {
        long long f = 0, b = 0, al = 0;
        PF[0] = PB[0] = PA[0] = 0;
        for (int l = 1; l <= L; ++l) {
            f += PF[l]; b += PB[l]; al += PA[l];
            // M * (time) and 2 (r-1) * (parameter bytes) must stay far from 2^63
            if (f + b >= PP_CAP62 / (M + 4 * D) || al >= PP_CAP62 / (2 * D)) { sh.fault = PP_FAULT_OVERFLOW; break; }
            PF[l] = f; PB[l] = b; PA[l] = al;
        }
        // int32 values if the largest stage term, the largest channel term and the largest
        // AllReduce remainder all stay below 2^30
        const long long lim = 1ll << 30;
        bool narrow = !sh.fault && M < (1 << 20);
        if (narrow && D > 1) {
            const long long bmin = (long long)sh.bmin;
            narrow = (long long)sh.bmax < lim / D &&
                     cdiv64((long long)sh.amax_f, bmin) + cdiv64((long long)sh.amax_b, bmin) < lim / M &&
                     2 * al / bmin + 1 < lim / 2;
        }
        narrow = narrow && f + b + 2 < lim / (2 * M);
        sh.wide = !narrow;
    }
    __syncthreads();
    if (blockIdx.x == 0) {
        if (!sh.fault)
            for (int l = tid; l <= L; l += B) {
                a.pre_out[l] = PF[l];
                a.pre_out[L1 + l] = PB[l];
                a.pre_out[2 * L1 + l] = PA[l];
            }
    }
    if (sh.fault) {
        // nothing can be planned: every (candidate, stage count) is marked as having no plan
        if (tid == 0 && blockIdx.x == 0) pp_raise(a.status, sh.fault);
        for (long long t = (long long)blockIdx.x * B + tid; t < a.N * D; t += (long long)gridDim.x * B)
            a.W_out[t] = PP_INF64;
        return;
    }
    if (sh.wide) prm_run<true>(a, smem, sh);
    else prm_run<false>(a, smem, sh);
}

// Row c = the ordering of lexicographic rank c among all D! (D <= 20).
__global__ __launch_bounds__(256) void k_all_orderings(int D, long long N, int *ord) {
    const long long c = (long long)blockIdx.x * 256 + threadIdx.x;
    if (c >= N) return;
    unsigned long long rem = (unsigned long long)c;
    unsigned used = 0;
    for (int n = 0; n < D; ++n) ord[c * D + n] = pp_unrank_next(D, n, rem, used);
}

// Workspace of pp_plan_replicated.
struct rep_layout {
    size_t slots_at, ord, pre, W, T, bounds, reps, part, total;
    int slots;
};

static rep_layout rep_layout_of(int L, int D, int64_t N) {
    rep_layout w;
    size_t off = 0;
    const size_t tri = (size_t)D * (D + 1) / 2;
    w.slots = (int)(N < 2560 ? N : 2560);  // 10 workgroups of 128 threads per compute unit
    w.slots_at = off; off += pp_align256((size_t)w.slots * prm_slot_bytes(L, D));
    w.ord = off;      off += pp_align256((size_t)N * D * 4);
    w.pre = off;      off += pp_align256((size_t)3 * (L + 1) * 8);
    w.W = off;        off += pp_align256((size_t)N * D * 8);
    w.T = off;        off += pp_align256((size_t)N * D * 8);
    w.bounds = off;   off += pp_align256((size_t)N * tri * 4);
    w.reps = off;     off += pp_align256((size_t)N * tri * 4);
    w.part = off;     off += pp_align256((size_t)1024 * 16);
    w.total = off;
    return w;
}

static bool rep_sizes_ok(int L, int D, int64_t N, const int32_t *orderings) {
    if (L < 1 || L > PP_MAX_LAYERS || D < 1 || D > 16 || N < 1) return false;
    if (prm_lds_bytes(L, D) > 64 * 1024) return false;
    if (!orderings) {
        int64_t f = 1;
        for (int i = 2; i <= D; ++i) f *= i;  // D <= 16: no overflow
        if (f != N) return false;
    }
    return true;
}

extern "C" size_t pp_workspace_bytes_replicated(int L, int D, int64_t N) {
    if (L < 1 || L > PP_MAX_LAYERS || D < 1 || D > 16 || N < 1) return 0;
    if (prm_lds_bytes(L, D) > 64 * 1024) return 0;
    return rep_layout_of(L, D, N).total;
}

extern "C" int pp_plan_replicated(int L, int D, int64_t N, int M, const int64_t *fwd_us,
                                  const int64_t *bwd_us, const int64_t *act_fwd_bytes,
                                  const int64_t *act_bwd_bytes, const int64_t *alpha_bytes,
                                  const int64_t *bw, const int32_t *orderings, pp_rep_result *out,
                                  int64_t *T_all, int64_t *W_all, int32_t *bounds_all,
                                  int32_t *reps_all, void *workspace, size_t workspace_bytes,
                                  int32_t *status, void *stream) {
    if (!rep_sizes_ok(L, D, N, orderings) || M < 1) return PP_ERR_INVALID_ARG;
    if (!fwd_us || !bwd_us || !act_fwd_bytes || !alpha_bytes || !bw || !out) return PP_ERR_INVALID_ARG;
    const rep_layout lay = rep_layout_of(L, D, N);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < lay.total) return PP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)workspace;
    const int32_t *ord = orderings;
    if (!ord) {
        int *list = (int *)(base + lay.ord);
        hipLaunchKernelGGL(k_all_orderings, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, D,
                           (long long)N, list);
        if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
        ord = list;
    }
    const int64_t *actb = act_bwd_bytes ? act_bwd_bytes : act_fwd_bytes;
    int64_t *W = W_all ? W_all : (int64_t *)(base + lay.W);
    int64_t *T = T_all ? T_all : (int64_t *)(base + lay.T);
    int32_t *bounds = bounds_all ? bounds_all : (int32_t *)(base + lay.bounds);
    int32_t *reps = reps_all ? reps_all : (int32_t *)(base + lay.reps);
    int64_t *pre = (int64_t *)(base + lay.pre);

    prm_args a;
    a.L = L; a.D = D; a.M = M; a.N = N;
    a.fwd = (const long long *)fwd_us; a.bwd = (const long long *)bwd_us;
    a.actf = (const long long *)act_fwd_bytes; a.actb = (const long long *)actb;
    a.alpha = (const long long *)alpha_bytes; a.bw = (const long long *)bw;
    a.ord = ord;
    a.scratch = base + lay.slots_at;
    a.slot_bytes = prm_slot_bytes(L, D);
    a.W_out = (long long *)W; a.bounds_out = bounds; a.reps_out = reps;
    a.pre_out = (long long *)pre;
    a.status = status;
    hipLaunchKernelGGL(k_prm, dim3(lay.slots), dim3(PRM_THREADS), prm_lds_bytes(L, D), st, a);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return pp_launch_rep_makespan(L, D, N, M, pre, pre + (L + 1), pre + 2 * (L + 1), act_fwd_bytes,
                                  actb, bw, ord, bounds, reps, W, T, status, base + lay.part,
                                  out, st);
}
