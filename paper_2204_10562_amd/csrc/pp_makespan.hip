// pp_schedule_makespan: per-iteration time of a plan under the pipeline execution scheduler
// (Alg. 1, Sec. IV-A), and the candidate arg-min of the SPP listing (Alg. 3).
//
// The scheduler's two phases collapse into a max-plus recurrence.  Its ordering phase moves
// every microbatch one block per sweep, so block j serves microbatch m = t - j + 1 in sweep
// t; each of the R = 2S-1 serial resources (stages, and one channel per stage pair for both
// directions) serves its items in (sweep, block) order, and an item starts when its
// microbatch has left block j-1 (which happened in sweep t-1) and the resource is idle:
//     fin_t[j] = max(fin_{t-1}[j-1], idle(resource of j)) + dur[j],
// where a resource's idle time is the latest finish of its two blocks j and 2R-j (finish
// times on one resource never decrease).  Within a sweep the forward block of a resource
// precedes its backward block.  All blocks of a sweep depend only on the sweep before (the
// anti-diagonal t = m + j - 1 of the (block, microbatch) grid), so one lane carries one
// candidate and all lanes run the same uniform loop.
//
// Two kernels: for S <= 16 the 4S-3 durations and finish times of a lane live in registers
// (blocks unrolled; for S <= 8 the block ranges of the ramp-up, steady or sliding-window and
// ramp-down sweeps are compile-time constants, otherwise every block is computed in every
// sweep and its update kept or dropped; 32-bit when the bound (M+4S-4) * largest block of
// Lemma 1 fits, else 64-bit, decided per wave; several microbatch counts run side by side,
// one wave each, in workgroups that share the gather of the block durations); for larger S
// they live in the lane's own LDS column.
// When asked to, each wave also reduces (T, candidate) to its minimum, and a one-workgroup
// kernel launched next reduces the per-wave minima to the winner record.
#include "pp_common.h"
#include "pp_dp_flat.h"

struct tc_pair { long long T, c; };

struct mk_args {
    int L, D, S, nM;
    int Ms[PP_MAX_M_LIST];  // microbatch counts; the plans are evaluated once per entry
    // k_makespan_regs: wave slot i (blockIdx.y * waves + wave) serves count Ms[order[i]]
    unsigned char order[PP_MAX_M_LIST];
    // k_makespan_regs8: a workgroup holds `groups` groups of waves, each group one wave per
    // microbatch count for its own 64 candidates; wave w of group g takes slot
    // (slot_perm >> 2 (4 g + w)) & 3 of its four
    int groups;
    unsigned slot_perm;
    // k_makespan_regs8: nonzero = blockIdx.z + 1 is the number of stages xi, the plan with xi
    // stages is read from the triangular bounds array and T goes to column xi-1 (S, bnd_off and
    // t_off are then ignored)
    int all_xi;
    // With all_xi and the library's own list of all D! orderings in lexicographic order:
    // share[xi] = (D - xi)! consecutive candidates share their first xi devices and with them
    // the plan of xi stages, so it is scheduled once per such block (share[xi] = 1: no sharing)
    long long share[9];
    long long N;
    const long long *PF, *PB, *XF, *XB;
    const int *orderings;  // NULL = all D! orderings, candidate index = lexicographic rank
    const int *bounds;
    long long *T_out;      // [nM][N]; may be NULL when only the winners are wanted
    // Where candidate c's data lie: devices at orderings[c*ord_stride + n], bounds at
    // bounds[c*bnd_stride + bnd_off + n], T of microbatch count q at
    // T_out[(q*N + c)*t_stride + t_off].  (ord_stride, bnd_stride, bnd_off, t_stride, t_off)
    // = (S, S, 0, 1, 0) for plain lists; the stage-count search evaluates the plans with S = xi
    // stages out of rows that hold search = S_max devices and all S_max plans.
    int ord_stride, bnd_off, t_off;
    long long bnd_stride, t_stride;
    // search > 0 (arg-min only): the N entries are (candidate, stage count) pairs, entry
    // i = c*search + xi-1; the record of the winner is decoded accordingly
    int search;
    int variant;  // k_makespan_variant only: PP_SCHED_*
    // k_makespan_mid / k_makespan_lds launched together without a header (17..32 stages, no
    // workspace): nonzero = every block of 64 candidates decides for itself which of the two
    // kernels schedules it (see mid_takes_block)
    int by_block;
    // workspace header with the largest time of the tables (NULL if there is none): lets every
    // wave of a launch take the same decision between 32-bit and 64-bit finish times
    const pp_ws_header *hdr;
    // k_makespan_regs8 inside pp_best_plan: nonzero = when no link's channel time depends on the
    // cut position and every finish time of the launch fits 32 bits (both read from hdr), the
    // partition DP kernel has left the plans to this kernel, which builds them in closed form
    // from the channel-free tables bfl (pp_dp_flat.h) and writes C_w [N] and bounds_w [N][S].
    // fuse_mmax: the largest microbatch count of the call (the DP kernel tests the same bound).
    int fuse, fuse_mmax, fuse_validate;
    const long long *bfl;
    long long *C_w;
    int *bounds_w;
    int32_t *status;
    // replicated stages (k_rep_makespan and the record of its arg-min; NULL otherwise): replica
    // counts laid out like bounds, prefix sums of the parameter sizes, activation sizes, the
    // bandwidth matrix, and W per (candidate, stage count) (PP_INF64 = no such plan)
    const int *reps;
    const long long *PA, *actf, *actb, *bw, *W;
    // k_makespan_regs<S> inside pp_best_plan: non-NULL = if the workspace header says that
    // candidates share their partition DP (pp_share.hip), this is the list of the candidates
    // that stand for all others; only they are scheduled (entry i by lane i of the launch), and
    // the slots of the partials no wave writes hold "none" already
    const int *rlist;
    pp_rep_result *rout;   // [nM] winner records with replica counts (instead of out)
    // arg-min (all NULL when not wanted)
    tc_pair *part;         // [nM][waves]: every wave's minimum, reduced by k_pick
    long long n_part;      // k_pick: partials per microbatch count
    const long long *C;
    pp_result *out;        // [nM]
};

__device__ __forceinline__ tc_pair tc_min(tc_pair a, tc_pair b) {
    return (b.T < a.T || (b.T == a.T && b.c < a.c)) ? b : a;
}

__device__ __forceinline__ tc_pair wave_tc_min(tc_pair v) {
    for (int off = 32; off; off >>= 1) {
        tc_pair o;
        o.T = __shfl_xor(v.T, off);
        o.c = __shfl_xor(v.c, off);
        v = tc_min(v, o);
    }
    return v;
}

// Checks candidate c's ordering and bounds and gathers its block durations through `put`
// (called as put(block j (1-based), duration)).  Returns fault bits; on a fault or for a
// dead lane all durations are 0.  `worst` gets the largest per-resource time f + b.
// ST > 0 fixes the number of stages at compile time (block numbers become constants).
// `last(F, B)` receives the last stage's forward and backward times separately.
// With parts > 1 only the stages n with n % parts == part are looked up (and reported through
// put/last); `worst` then covers those stages only.
template <int ST, typename Put, typename Last>
__device__ __forceinline__ int gather_durations(const mk_args &a, long long c, bool live,
                                                long long &worst, Put put, Last last,
                                                int part = 0, int parts = 1) {
    const int S = ST ? ST : a.S, L = a.L, D = a.D, R = 2 * S - 1;
    // (k_makespan_regs8 with all_xi: the plan with ST stages of the triangular array)
    const int bnd_off = (ST && a.all_xi) ? ST * (ST - 1) / 2 : a.bnd_off;
    int fault = 0;
    if (live) {
        if (a.orderings) {
            for (int n = 0; n < S; ++n) {
                int d = a.orderings[c * a.ord_stride + n];
                bool bad = d < 0 || d >= D;
                for (int q = 0; q < n; ++q) bad |= (a.orderings[c * a.ord_stride + q] == d);
                if (bad) fault |= PP_FAULT_ORDERING;
            }
        }
        // (a bad ordering is reported alone: its plan is not looked at)
        int prev = 0, fb = 0;
        for (int n = 0; n < S; ++n) {
            int e = a.bounds[c * a.bnd_stride + bnd_off + n];
            if (e <= prev || e > L) fb = PP_FAULT_BOUNDS;
            prev = e;
        }
        if (prev != L) fb = PP_FAULT_BOUNDS;
        fault = fault ? fault : fb;
    }
    worst = 0;
    unsigned long long rem = (unsigned long long)(live ? c : 0);
    unsigned used = 0;
    int e_prev = 0, o_prev = 0;
#pragma unroll
    for (int n = 0; n < S; ++n) {
        long long F = 0, Bk = 0, cf = 0, cb = 0;
        if (live && !fault) {
            int o_n = a.orderings ? a.orderings[c * a.ord_stride + n] : pp_unrank_next(D, n, rem, used);
            int e = a.bounds[c * a.bnd_stride + bnd_off + n];
            if (parts == 1 || n % parts == part) {
                F = a.PF[e] - a.PF[e_prev];
                Bk = a.PB[e] - a.PB[e_prev];
                if (n) {
                    size_t at = ((size_t)o_prev * D + o_n) * L + (size_t)(e_prev - 1);
                    cf = a.XF[at];
                    cb = a.XB[at];
                }
            }
            e_prev = e;
            o_prev = o_n;
        }
        if (parts != 1 && n % parts != part) continue;
        long long w = F + Bk > cf + cb ? F + Bk : cf + cb;
        worst = w > worst ? w : worst;
        const int r = 2 * n + 1;  // stage n is resource 2n+1, channel n is resource 2n
        if (n == S - 1) {
            put(R, F + Bk);  // merged forward+backward block of the last stage
            last(F, Bk);
        } else {
            put(r, F);
            put(2 * R - r, Bk);
        }
        if (n) {
            put(r - 1, cf);
            put(2 * R - (r - 1), cb);
        }
    }
    return fault;
}

template <int ST, typename Put>
__device__ __forceinline__ int gather_durations(const mk_args &a, long long c, bool live,
                                                long long &worst, Put put) {
    return gather_durations<ST>(a, c, live, worst, put, [](long long, long long) {});
}

// The schedule is no longer than (M + 4S - 4) * C (Lemma 1): fault if that bound reaches 2^62.
__device__ __forceinline__ int overflow_fault(long long worst, int M, int S) {
    return worst > (PP_CAP62 - 1) / ((long long)M + 4 * S - 4) ? PP_FAULT_OVERFLOW : 0;
}

// Writes T of microbatch count q, raises faults, and (if wanted) leaves the wave's minimum in
// its slot of the partials; k_pick, launched next on the same stream, reduces the partials.
// (Plain stores and a kernel boundary: earlier versions let the last wave to arrive do the
// final reduction, but the returned atomics and arrival counters that needs cost more than
// the schedule itself once a launch has thousands of waves.)
__device__ __forceinline__ void emit(const mk_args &a, int q, long long c, bool live, int fault,
                                     long long T, long long wave_id, long long n_waves, int t_off) {
    if (live) {
        if (fault) { T = PP_INF64; pp_raise(a.status, fault); }
        if (a.T_out) a.T_out[((long long)q * a.N + c) * a.t_stride + t_off] = T;
    }
    if (!a.part) return;
    tc_pair v = {live ? T : PP_INF64, live ? c : INT64_MAX};
    v = wave_tc_min(v);
    if ((threadIdx.x & 63) == 0 && wave_id < n_waves) a.part[(long long)q * n_waves + wave_id] = v;
}

// The winner record of microbatch count q from the minimum w over all entries.
__device__ __forceinline__ void write_winner(const mk_args &a, int q, tc_pair w, int lane) {
    const int S = a.S;
    const bool none = w.T == PP_INF64;
    // the winner: candidate c with xi stages, its C at C[at_c], its bounds from bounds[at_b]
    long long c = w.c, at_c = w.c, at_b = w.c * a.bnd_stride + a.bnd_off;
    int xi = S;
    if (a.search && !none) {
        c = w.c / a.search;
        xi = (int)(w.c - c * a.search) + 1;
        at_b = c * ((long long)a.search * (a.search + 1) / 2) + xi * (xi - 1) / 2;
    }
    if (a.rout) {
        // plan with replicated stages: xi bounds and replica counts, all D devices by rank
        pp_rep_result *out = a.rout + q;
        if (lane == 0) {
            out->best_index = none ? -1 : c;
            out->T = w.T;
            out->W = none ? PP_INF64 : a.C[at_c];
            out->S = none ? 0 : xi;
        }
        const bool in = lane < xi && !none;
        out->bounds[lane] = in ? a.bounds[at_b + lane] : 0;
        out->reps[lane] = in ? a.reps[at_b + lane] : 0;
        out->order[lane] = (lane < a.D && !none) ? a.orderings[c * a.ord_stride + lane] : 0;
        return;
    }
    pp_result *out = a.out + q;
    if (lane == 0) {
        out->best_index = none ? -1 : c;
        out->T = w.T;
        out->C = none ? PP_INF64 : a.C[at_c];
        out->S = xi;
    }
    // lane n writes bound n and device n (lanes xi.. write zeros)
    int b = 0, o = 0;
    if (lane < xi && !none) {
        b = a.bounds[at_b + lane];
        if (a.orderings) {
            o = a.orderings[c * a.ord_stride + lane];
        } else {
            unsigned long long rem = (unsigned long long)c;
            unsigned used = 0;
            for (int n = 0; n <= lane; ++n) o = pp_unrank_next(a.D, n, rem, used);
        }
    }
    out->bounds[lane] = b;
    out->order[lane] = o;
}

// One workgroup per microbatch count: the minimum (T, index) of its n_part partials, lowest
// index on ties, and the winner record.
__global__ __launch_bounds__(256) void k_pick(mk_args a) {
    __shared__ tc_pair sh[4];
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const tc_pair *part = a.part + (long long)q * a.n_part;
    tc_pair w = {PP_INF64, INT64_MAX};
    // four loads in flight per thread: the partials come straight from the kernel before, so
    // each round is a trip to memory
    const tc_pair none = {PP_INF64, INT64_MAX};
    for (long long i = tid; i < a.n_part; i += 1024) {
        tc_pair p0 = part[i];
        tc_pair p1 = i + 256 < a.n_part ? part[i + 256] : none;
        tc_pair p2 = i + 512 < a.n_part ? part[i + 512] : none;
        tc_pair p3 = i + 768 < a.n_part ? part[i + 768] : none;
        w = tc_min(tc_min(w, p0), tc_min(p1, tc_min(p2, p3)));
    }
    w = wave_tc_min(w);
    if (lane == 0) sh[tid >> 6] = w;
    __syncthreads();
    if (tid < 64) {
        w = tc_min(tc_min(sh[0], sh[1]), tc_min(sh[2], sh[3]));
        write_winner(a, q, w, lane);
    }
}

static int launch_pick(mk_args a, int nM, long long n_part, hipStream_t st) {
    a.n_part = n_part;
    hipLaunchKernelGGL(k_pick, dim3(nM), dim3(256), 0, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

// ---------------------------------------------------------------- registers, S <= 16

// med3(old, fresh, sel) for 0 <= old <= fresh < 2^31: fresh if the scalar sel is all ones, old if it is 0.
__device__ __forceinline__ int keep_or_take(int old, int fresh, unsigned sel) {
    int r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(old), "v"(fresh), "s"(sel));
    return r;
}
__device__ __forceinline__ long long keep_or_take(long long old, long long fresh, unsigned sel) {
    return sel ? fresh : old;
}

// One sweep restricted to blocks LO..HI (compile-time), no validity tests.
template <int S, typename V, int LO, int HI>
__device__ __forceinline__ void sweep_blocks(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1]) {
    constexpr int R = 2 * S - 1, J = 2 * R - 1;
    const V finR_prev = fin[R];
    // forward blocks and the merged block R, descending so that fin[j-1] is still the
    // previous sweep's value
#pragma unroll
    for (int j = R; j >= 1; --j) {
        if (j < LO || j > HI) continue;
        V idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
        V ready = j > 1 ? fin[j - 1] : (V)0;
        fin[j] = (idle > ready ? idle : ready) + dur[j];
    }
    // backward blocks: the resource may just have been used by this sweep's forward block
#pragma unroll
    for (int j = J; j >= R + 1; --j) {
        if (j < LO || j > HI) continue;
        V idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
        V ready = j == R + 1 ? finR_prev : fin[j - 1];
        fin[j] = (idle > ready ? idle : ready) + dur[j];
    }
}

template <int S, typename V, int T>
__device__ __forceinline__ void ramp_up(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1]) {
    if constexpr (T <= 4 * S - 4) {
        sweep_blocks<S, V, 1, T>(fin, dur);
        ramp_up<S, V, T + 1>(fin, dur);
    }
}

template <int S, typename V, int U>
__device__ __forceinline__ void ramp_down(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1]) {
    if constexpr (U <= 4 * S - 4) {
        sweep_blocks<S, V, U + 1, 4 * S - 3>(fin, dur);
        ramp_down<S, V, U + 1>(fin, dur);
    }
}

// All M + 4S - 4 sweeps with the finish times in registers; returns the finish of the last
// backward block on stage 0.  Block j works in sweep t iff t-M+1 <= j <= t.  When the
// pipeline fills completely (M >= J-1) the sweeps split into a ramp-up (blocks 1..t), a
// steady phase (all blocks) and a ramp-down (blocks t-M+1..J) whose block ranges are known at
// compile time.  A shorter pipeline still has such a ramp-up (its first M sweeps) and ramp-down
// (its last M-1); in the sweeps between them, and in every sweep for S > 8 (where unrolling
// every sweep would be too much code), every block is computed and the update is kept or
// dropped by a select: with 32-bit times a median of three against a per-block scalar that is
// 0 or all ones (finish times never decrease, so med3(old, new, ~0) = new and
// med3(old, new, 0) = old), with 64-bit times a per-lane compare.
// `result(fin)` turns the final finish times into the value returned.
// Sweep t with every block computed and the update of the blocks outside [t-M+1, t] dropped.
template <int S, typename V>
__device__ __forceinline__ void sweep_selected(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1], int t, int M) {
    constexpr int R = 2 * S - 1, J = 2 * R - 1;
    const V finR_prev = fin[R];
    if constexpr (sizeof(V) == 4) {
        // bit j of `act`: block j works in this sweep
        const int jlo = t - M + 1 > 1 ? t - M + 1 : 1, jhi = t < J ? t : J;
        const unsigned long long act = ((2ull << jhi) - 1) & ~((1ull << jlo) - 1);
        // groups of G blocks without an active one are skipped altogether
        constexpr int G = 5;
#pragma unroll
        for (int jh = R; jh >= 1; jh -= G) {
            const int jl = jh - G + 1 > 1 ? jh - G + 1 : 1;
            if (!(act & (((2ull << jh) - 1) & ~((1ull << jl) - 1)))) continue;
#pragma unroll
            for (int j = jh; j >= jl; --j) {
                V idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
                V ready = j > 1 ? fin[j - 1] : (V)0;
                V nv = (idle > ready ? idle : ready) + dur[j];
                fin[j] = keep_or_take(fin[j], nv, (act >> j) & 1 ? ~0u : 0u);
            }
        }
#pragma unroll
        for (int jh = J; jh >= R + 1; jh -= G) {
            const int jl = jh - G + 1 > R + 1 ? jh - G + 1 : R + 1;
            if (!(act & (((2ull << jh) - 1) & ~((1ull << jl) - 1)))) continue;
#pragma unroll
            for (int j = jh; j >= jl; --j) {
                V idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
                V ready = j == R + 1 ? finR_prev : fin[j - 1];
                V nv = (idle > ready ? idle : ready) + dur[j];
                fin[j] = keep_or_take(fin[j], nv, (act >> j) & 1 ? ~0u : 0u);
            }
        }
    } else {
        // j is in [t-M+1, t] iff (unsigned)(j - (t-M+1)) <= M-1; kept in a vector register so
        // that the tests run on the vector unit next to the arithmetic
        const unsigned width = (unsigned)(M - 1);
        int jlo = t - M + 1;
        asm volatile("" : "+v"(jlo));
#pragma unroll
        for (int j = R; j >= 1; --j) {
            V idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
            V ready = j > 1 ? fin[j - 1] : (V)0;
            V nv = (idle > ready ? idle : ready) + dur[j];
            fin[j] = (unsigned)(j - jlo) <= width ? nv : fin[j];
        }
#pragma unroll
        for (int j = J; j >= R + 1; --j) {
            V idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
            V ready = j == R + 1 ? finR_prev : fin[j - 1];
            V nv = (idle > ready ? idle : ready) + dur[j];
            fin[j] = (unsigned)(j - jlo) <= width ? nv : fin[j];
        }
    }
}

// The first M sweeps of a pipeline that never fills (M <= J-2): blocks 1..t.
template <int S, typename V, int T>
__device__ __forceinline__ void ramp_up_to(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1], int M) {
    if constexpr (T <= 4 * S - 5) {
        if (T > M) return;
        sweep_blocks<S, V, 1, T>(fin, dur);
        ramp_up_to<S, V, T + 1>(fin, dur, M);
    }
}

// The last sweeps of a pipeline, blocks U+1..J for every U+1 >= lo.
template <int S, typename V, int U>
__device__ __forceinline__ void ramp_down_from(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1], int lo) {
    if constexpr (U <= 4 * S - 4) {
        if (U + 1 >= lo) sweep_blocks<S, V, U + 1, 4 * S - 3>(fin, dur);
        ramp_down_from<S, V, U + 1>(fin, dur, lo);
    }
}

// Sweeps M+1..J of a pipeline that never fills, for a microbatch count known at compile time:
// the window of M blocks moves up by one block per sweep.
template <int S, typename V, int M, int T>
__device__ __forceinline__ void slide_window(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1]) {
    if constexpr (T <= 4 * S - 3) {
        sweep_blocks<S, V, T - M + 1, T>(fin, dur);
        slide_window<S, V, M, T + 1>(fin, dur);
    }
}

// Picks the instance of slide_window for the run-time microbatch count m (1 <= m <= J-2).
template <int S, typename V, int M>
__device__ __forceinline__ void slide_window_for(V (&fin)[4 * S - 3 + 1], const V (&dur)[4 * S - 3 + 1], int m) {
    if constexpr (M <= 4 * S - 5) {
        if (m == M) {
            slide_window<S, V, M, M + 1>(fin, dur);
            return;
        }
        slide_window_for<S, V, M + 1>(fin, dur, m);
    }
}

template <int S, typename V, typename Result>
__device__ __forceinline__ long long sweep_regs(const long long (&dur64)[4 * S - 3 + 1], int M, Result result) {
    constexpr int R = 2 * S - 1, J = 2 * R - 1;
    V dur[J + 1], fin[J + 1];
#pragma unroll
    for (int j = 1; j <= J; ++j) { dur[j] = (V)dur64[j]; fin[j] = 0; }
    dur[0] = fin[0] = 0;
    if constexpr (S <= 8) {
        if (M >= J - 1) {
            ramp_up<S, V, 1>(fin, dur);
            for (int t = J; t <= M; ++t) sweep_blocks<S, V, 1, J>(fin, dur);
            ramp_down<S, V, 1>(fin, dur);
        } else {
            ramp_up_to<S, V, 1>(fin, dur, M);                                   // sweeps 1..M
            if constexpr (sizeof(V) == 4) slide_window_for<S, V, 1>(fin, dur, M);       // sweeps M+1..J
            else for (int t = M + 1; t <= J; ++t) sweep_selected<S, V>(fin, dur, t, M);
            ramp_down_from<S, V, 1>(fin, dur, J - M + 2);                       // sweeps J+1..J+M-1
        }
        return result(fin);
    }
    const int sweeps = M + 2 * R - 2;
    for (int t = 1; t <= sweeps; ++t) sweep_selected<S, V>(fin, dur, t, M);
    return result(fin);
}

// Microbatch counts handled by one group of waves of k_makespan_regs (one wave each), and the
// most groups a workgroup of k_makespan_regs8 holds.
#define MK_REGS_WAVES 4
#define MK_REGS_GROUPS 3

// LDS the fused gather needs: per group, J rows of 64 int32 durations and one row of 64 int64
// per wave (only when a group has several waves), then the tables: B and A of the channel-free
// program, PF, PB, and the forward and backward channel time of every link.
__host__ __device__ static inline size_t mk_fuse_exchange_bytes(int S, int nw, int G) {
    return nw > 1 ? (size_t)G * ((size_t)(4 * S - 3) * 64 * 4 + (size_t)nw * 64 * 8) : 0;
}
__host__ __device__ static inline size_t mk_fuse_lds_bytes(int L, int D, int S, int nw, int G) {
    return mk_fuse_exchange_bytes(S, nw, G) + pp_flat_table_bytes(L, S) + (size_t)2 * (L + 1) * 8 +
           (size_t)2 * D * D * 8;
}

// The gather of regs_body when the plans are not in memory yet (a.fuse): if the tables say so
// (see mk_args), every lane builds its candidate's plan in closed form from tables staged in
// LDS - W[n][l] = max(largest channel time so far, channel-free cell), lowest split from the
// channel-free split table or by a search in the prefix sums - and takes the block durations
// from LDS as well, so that the whole gather costs one trip to memory.  Returns false (nothing
// done) if this launch reads its plans from memory.  Must be entered by whole workgroups.
template <int S>
__device__ __forceinline__ bool fused_gather(const mk_args &a, long long c, bool live, int g, int w,
                                             int nw, int G, long long (&dur)[4 * S - 3 + 1],
                                             long long &worst, int &fault) {
    constexpr int R = 2 * S - 1, J = 4 * S - 3;
    extern __shared__ __align__(16) unsigned char fsm[];
    const int L = a.L, D = a.D, nP = L + 1, tid = threadIdx.x, lane = tid & 63;
    // requests first: header, this lane's row, the tables (8 pieces of 16 bytes per thread and
    // pass; contiguous in the workspace as B then A), PF, PB, and the links' channel times
    const unsigned flat_w = a.hdr->flat[lane];
    unsigned long long vmax = a.hdr->pmax[lane];
    int row[S];
#pragma unroll
    for (int n = 0; n < S; ++n) row[n] = live ? a.orderings[c * a.ord_stride + n] : 0;
    const size_t tab = pp_flat_table_bytes(L, S);
    unsigned char *tbase = fsm + mk_fuse_exchange_bytes(S, nw, G);
    long long *sB = (long long *)tbase;
    int *sA = (int *)(sB + (size_t)S * nP);
    long long *sPF = (long long *)(tbase + tab), *sPB = sPF + nP, *sxf = sPB + nP, *sxb = sxf + D * D;
    const int n16 = (int)(tab / 16), T = blockDim.x;
    int4 first[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) first[u] = tid + u * T < n16 ? ((const int4 *)a.bfl)[tid + u * T] : make_int4(0, 0, 0, 0);
    // (what the first pass of the loops below stores)
    long long pf0 = tid <= L ? a.PF[tid] : 0, pb0 = tid <= L ? a.PB[tid] : 0;
    long long xf0 = (tid < D * D && L > 1) ? a.XF[(size_t)tid * L] : 0, xb0 = (tid < D * D && L > 1) ? a.XB[(size_t)tid * L] : 0;
    // (lane b holds the largest time of pack block b: all below the limit = their maximum is)
    const bool fused = __ballot(flat_w != 0) == ~0ull &&
                       !__ballot(vmax > 0x7fffffffull / (unsigned long long)(a.fuse_mmax + 4 * S - 4));
    if (!fused) return false;
#pragma unroll
    for (int u = 0; u < 8; ++u)
        if (tid + u * T < n16) ((int4 *)sB)[tid + u * T] = first[u];
    for (int base = 8 * T; base < n16; base += 8 * T) {  // (narrow workgroups: further passes)
        int4 more[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            more[u] = base + tid + u * T < n16 ? ((const int4 *)a.bfl)[base + tid + u * T] : make_int4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (base + tid + u * T < n16) ((int4 *)sB)[base + tid + u * T] = more[u];
    }
    for (int i = tid; i <= L; i += T) {
        sPF[i] = i == tid ? pf0 : a.PF[i];
        sPB[i] = i == tid ? pb0 : a.PB[i];
    }
    for (int i = tid; i < D * D; i += T) {
        sxf[i] = i == tid ? xf0 : (L > 1 ? a.XF[(size_t)i * L] : 0);
        sxb[i] = i == tid ? xb0 : (L > 1 ? a.XB[(size_t)i * L] : 0);
    }
    __syncthreads();

    // a caller's row is checked here (the DP kernel has not looked at it)
    bool bad = false;
    if (a.fuse_validate && live) {
#pragma unroll
        for (int n = 0; n < S; ++n) {
            bad |= row[n] < 0 || row[n] >= D;
#pragma unroll
            for (int q = 0; q < n; ++q) bad |= row[q] == row[n];
        }
    }
    fault = bad ? PP_FAULT_ORDERING : 0;
    if (bad) {
#pragma unroll
        for (int n = 0; n < S; ++n) row[n] = 0;
    }
    // prefix maxima of the channel times, then the plan from (S-1, L) downwards
    long long m[S];
    int link[S];
    m[0] = 0;
    link[0] = 0;
#pragma unroll
    for (int n = 1; n < S; ++n) {
        link[n] = row[n - 1] * D + row[n];
        m[n] = sxf[link[n]] + sxb[link[n]];
    }
#pragma unroll
    for (int n = 1; n < S; ++n) m[n] = m[n] > m[n - 1] ? m[n] : m[n - 1];
    int e[S];
    long long Cval = sB[L];  // S == 1: P[L]
    e[S - 1] = L;
    const int steps = pp_flat_steps(L);
#pragma unroll
    for (int n = S - 1; n >= 1; --n) {
        const long long bn = sB[(size_t)n * nP + e[n]];
        int r = sA[(size_t)n * nP + e[n]];
        if (n == S - 1) Cval = m[n] > bn ? m[n] : bn;
        if (m[n] > bn) {  // the channels bind: the longest last stage that fits in m_n
            const long long t = sB[e[n]] - m[n];
            int pos = 0;
            for (int st = 1 << (steps - 1); st; st >>= 1) {
                const int idx = pos + st - 1;
                pos += sB[idx <= L ? idx : L] < t ? st : 0;
            }
            r = pos < L ? pos : L;
            r = r > n ? r : n;
        }
        e[n - 1] = r;
    }
    // the plan goes to memory once per candidate (the winner's record is read from there)
    if (w == 0 && live) {
        a.C_w[c] = bad ? PP_INF64 : Cval;
        int *bo = a.bounds_w + c * S;
        if (S == 8) {
            *(int4 *)bo = bad ? make_int4(0, 0, 0, 0) : make_int4(e[0], e[1], e[2], e[3]);
            *(int4 *)(bo + 4) = bad ? make_int4(0, 0, 0, 0) : make_int4(e[4], e[5], e[6], e[7]);
        } else {
#pragma unroll
            for (int n = 0; n < S; ++n) bo[n] = bad ? 0 : e[n];
        }
    }
    // block durations of this wave's share of the stages (all of them for a single wave)
    int *xd = (int *)fsm + (size_t)g * ((size_t)J * 64 + (size_t)nw * 128) + lane;  // [J][64] int32, then [nw][64] int64
    long long mine = 0;
    const bool use = live && !bad;
#pragma unroll
    for (int n = 0; n < S; ++n) {
        if (nw > 1 && n % nw != w) continue;
        const int e0 = n ? e[n - 1] : 0;
        long long F = sPF[e[n]] - sPF[e0], Bk = sPB[e[n]] - sPB[e0], cf = 0, cb = 0;
        if (n) { cf = sxf[link[n]]; cb = sxb[link[n]]; }
        if (!use) F = Bk = cf = cb = 0;
        const long long wn = F + Bk > cf + cb ? F + Bk : cf + cb;
        mine = wn > mine ? wn : mine;
        const int r = 2 * n + 1;
        auto put = [&](int j, long long d) {
            if (nw > 1) xd[(j - 1) * 64] = (int)d;
            else dur[j] = d;
        };
        if (n == S - 1) put(R, F + Bk);
        else { put(r, F); put(2 * R - r, Bk); }
        if (n) { put(r - 1, cf); put(2 * R - (r - 1), cb); }
    }
    worst = mine;
    if (nw > 1) {
        long long *xw = (long long *)((int *)fsm + (size_t)g * ((size_t)J * 64 + (size_t)nw * 128) + (size_t)J * 64);
        xw[w * 64 + lane] = mine;
        __syncthreads();
#pragma unroll
        for (int j = 1; j <= J; ++j) dur[j] = xd[(j - 1) * 64];
        worst = 0;
        for (int v = 0; v < nw; ++v) {
            const long long o = xw[v * 64 + lane];
            worst = o > worst ? o : worst;
        }
    }
    dur[0] = 0;
    return true;
}

// One wave per (64 candidates, microbatch count).  The waves of a workgroup serve the same 64
// candidates for up to MK_REGS_WAVES counts: the scattered table lookups of the gather, which
// cost more than the schedule itself for small M, are split between them by stage and
// exchanged through LDS (dynamic, (J + 1 + waves) * 64 * 8 bytes; none for a single wave).
template <int S, bool SHARE = false, bool LISTED = false>
__device__ __forceinline__ void regs_body(const mk_args &a) {
    constexpr int R = 2 * S - 1, J = 4 * S - 3;
    extern __shared__ __align__(16) long long sh_all[];  // per group: [J+1][64] durations, [nw][64] worst
    long long *sh_dur = sh_all;
    const int lane = threadIdx.x & 63;
    // wave w of nw in group g of G: a group serves 64 candidates
    const int G = a.groups, nw = (int)(blockDim.x >> 6) / G;
    const int wall = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = wall / nw, w = wall - g * nw;
    const long long group = (long long)blockIdx.x * G + g;
    // one lane per candidate, or per block of `f` candidates that share this plan
    const long long f = SHARE ? a.share[S <= 8 ? S : 0] : 1;
    if (SHARE && (long long)blockIdx.x * 64 * f >= a.N) return;  // (the whole workgroup; G = 1)
    long long c = (group * 64 + lane) * f;
    bool live = c < a.N;
    if constexpr (LISTED) {
        if (a.rlist && a.hdr->share_active) {
            const long long todo = a.hdr->share_nreps;
            if (group * 64 >= todo) return;  // (the whole workgroup: G = 1)
            live = group * 64 + lane < todo;
            c = live ? pp_share_at(a.hdr, a.rlist, a.N, group * 64 + lane) : 0;
        }
    }
    sh_dur += (size_t)g * (J + 1 + nw) * 64;
    long long dur[J + 1];
    long long worst;
    int fault;
    bool gathered = false;
    if constexpr (!SHARE && !(LISTED && S <= 8) && S >= 2 && S <= 8) {
        if (a.fuse) gathered = fused_gather<S>(a, c, live, g, w, nw, G, dur, worst, fault);
    }
    if (gathered) {
        // durations, worst and fault are set
    } else if (nw == 1) {
        fault = gather_durations<S>(a, c, live, worst, [&](int j, long long d) { dur[j] = d; });
    } else {
        long long mine;
        fault = gather_durations<S>(a, c, live, mine,
                                    [&](int j, long long d) { sh_dur[j * 64 + lane] = d; },
                                    [](long long, long long) {}, w, nw);
        sh_dur[(J + 1) * 64 + w * 64 + lane] = mine;
        __syncthreads();
#pragma unroll
        for (int j = 1; j <= J; ++j) dur[j] = sh_dur[j * 64 + lane];
        worst = 0;
        for (int v = 0; v < nw; ++v) {
            const long long o = sh_dur[(J + 1) * 64 + v * 64 + lane];
            worst = o > worst ? o : worst;
        }
    }
    // The wave's microbatch count: the counts run side by side, not in a loop.
    // Which wave of a group takes which count differs between the groups of a workgroup
    // (slot_perm, chosen by the host): see launch_regs.
    const int ws = (a.slot_perm >> (2 * (g * 4 + w))) & 3;
    const int slot = blockIdx.y * nw + ws;
    if (slot >= a.nM) return;
    // (selected with constant indices: a run-time index into the argument struct can make the
    // compiler keep a copy of all of it in scratch memory, which cost 12 us per launch)
    int q = 0, M = 1;
#pragma unroll
    for (int i = 0; i < PP_MAX_M_LIST; ++i) q = i == slot ? (int)a.order[i] : q;
#pragma unroll
    for (int i = 0; i < PP_MAX_M_LIST; ++i) M = i == q ? a.Ms[i] : M;
    const int fq = (live && !fault) ? overflow_fault(worst, M, S) : fault;
    // 32-bit arithmetic if no finish time of any lane can reach 2^31
    const bool narrow = fq || !live || worst <= (long long)0x7fffffff / ((long long)M + 4 * S - 4);
    // T is the finish of the last backward block on stage 0
    long long T;
    if (__all(narrow)) T = sweep_regs<S, int>(dur, M, [](const int (&fin)[J + 1]) { return (long long)fin[J]; });
    else T = sweep_regs<S, long long>(dur, M, [](const long long (&fin)[J + 1]) { return fin[J]; });
    if (!SHARE || f == 1) {
        emit(a, q, c, live, fq, T, group, (a.N + 63) / 64, a.all_xi ? S - 1 : a.t_off);
        return;
    }
    // every candidate of the lane's block gets the block's T
    if (live && fq) pp_raise(a.status, fq);
    if (fq) T = PP_INF64;
    for (long long i = 0; i < f; ++i)
        if (c + i < a.N) a.T_out[((long long)q * a.N + c + i) * a.t_stride + (S - 1)] = T;
}

// 9 <= S <= 16: one kernel per S.
template <int S>
__global__ __launch_bounds__(64 * MK_REGS_WAVES) void k_makespan_regs(mk_args a) {
    regs_body<S, false, true>(a);
}

// S <= 8: one kernel for all of them, so that the stage-count search can evaluate the plans of
// every stage count xi = 1..S in a single launch (blockIdx.z = xi - 1) instead of S launches
// whose fixed costs add up.
__global__ __launch_bounds__(64 * MK_REGS_WAVES * MK_REGS_GROUPS) void k_makespan_regs8(mk_args a) {
    // (the arguments stay untouched: a modified copy would live in scratch memory)
    switch (a.all_xi ? (int)blockIdx.z + 1 : a.S) {
        case 1: regs_body<1>(a); break;
        case 2: regs_body<2>(a); break;
        case 3: regs_body<3>(a); break;
        case 4: regs_body<4>(a); break;
        case 5: regs_body<5>(a); break;
        case 6: regs_body<6>(a); break;
        case 7: regs_body<7>(a); break;
        case 8: regs_body<8>(a); break;
    }
}

// The same over the list of representatives (see mk_args::rlist; always one group per
// workgroup).  A kernel of its own so that the plain one stays as lean as it is.
__global__ __launch_bounds__(64 * MK_REGS_WAVES) void k_makespan_regs8_listed(mk_args a) {
    switch (a.all_xi ? (int)blockIdx.z + 1 : a.S) {
        case 1: regs_body<1, false, true>(a); break;
        case 2: regs_body<2, false, true>(a); break;
        case 3: regs_body<3, false, true>(a); break;
        case 4: regs_body<4, false, true>(a); break;
        case 5: regs_body<5, false, true>(a); break;
        case 6: regs_body<6, false, true>(a); break;
        case 7: regs_body<7, false, true>(a); break;
        case 8: regs_body<8, false, true>(a); break;
    }
}

// The same for the stage-count search over the library's own lexicographic list of all D!
// orderings (always with all_xi): plans shared by blocks of consecutive candidates are
// scheduled once per block.  A kernel of its own so that the plain one stays as lean as it is.
__global__ __launch_bounds__(64 * MK_REGS_WAVES) void k_makespan_regs8_shared(mk_args a) {
    switch ((int)blockIdx.z + 1) {
        case 1: regs_body<1, true>(a); break;
        case 2: regs_body<2, true>(a); break;
        case 3: regs_body<3, true>(a); break;
        case 4: regs_body<4, true>(a); break;
        case 5: regs_body<5, true>(a); break;
        case 6: regs_body<6, true>(a); break;
        case 7: regs_body<7, true>(a); break;
        case 8: regs_body<8, true>(a); break;
    }
}

// ---------------------------------------------------------------- replicated stages, S <= 16

__device__ __forceinline__ long long ceil_div64(long long x, long long y) { return x / y + (x % y != 0); }

// Plans with replicated stages (Sec. III-B): stage s runs on reps[s] GPUs of consecutive ranks,
// a replica takes ceil(p / k) per microbatch, a transfer between stages of k' and k replicas
// ceil(d / (k' k min b)) with the minimum over the links between the two GPU sets, and a
// replicated stage ends with a ring AllReduce of ceil(2 (k-1) sum alpha / (k min b)) (Eq. 1)
// that starts when its last backward pass has finished.  T is the later of the last backward
// block on stage 0 and the end of the last AllReduce (Eq. 2).  One lane per candidate; the
// plan with S stages of candidate c is read from the triangular arrays.
template <int S>
__global__ __launch_bounds__(64) void k_rep_makespan(mk_args a) {
    constexpr int R = 2 * S - 1, J = 4 * S - 3;
    const int lane = threadIdx.x, L = a.L, D = a.D;
    const long long c = (long long)blockIdx.x * 64 + lane;
    const bool live = c < a.N;
    const int M = a.Ms[0];
    long long dur[J + 1], A[S];
    long long worst = 0, amax = 0;
    int fault = 0;
    const bool none = live && a.W[c * a.t_stride + a.t_off] == PP_INF64;  // no plan with S stages
    const bool work = live && !none;
    const int *bd = a.bounds + c * a.bnd_stride + a.bnd_off;
    const int *rp = a.reps + c * a.bnd_stride + a.bnd_off;
    const int *o = a.orderings + c * a.ord_stride;
    if (work) {
        int prev = 0, used = 0;
        for (int s = 0; s < S; ++s) {
            int e = bd[s], k = rp[s];
            if (e <= prev || e > L || k < 1 || k > D) fault |= PP_FAULT_BOUNDS;
            prev = e;
            used += k;
        }
        if (prev != L || used != D) fault |= PP_FAULT_BOUNDS;
        for (int n = 0; n < D; ++n) {
            int d = o[n];
            bool bad = d < 0 || d >= D;
            for (int q = 0; q < n; ++q) bad |= (o[q] == d);
            if (bad) fault |= PP_FAULT_ORDERING;
        }
    }
    const bool ok = work && !fault;
    int e0 = 0, n = 0, kprev = 0;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        long long F = 0, Bk = 0, cf = 0, cb = 0, As = 0;
        if (ok) {
            const int e = bd[s], k = rp[s];
            F = ceil_div64(a.PF[e] - a.PF[e0], k);
            Bk = ceil_div64(a.PB[e] - a.PB[e0], k);
            if (k > 1) {
                long long m = PP_INF64;
                for (int u = n; u < n + k; ++u)
                    for (int v = n; v < n + k; ++v)
                        if (u != v) {
                            long long x = a.bw[(size_t)o[u] * D + o[v]];
                            m = x < m ? x : m;
                        }
                As = ceil_div64(2 * (long long)(k - 1) * (a.PA[e] - a.PA[e0]), (long long)k * m);
            }
            if (s) {
                long long mf = PP_INF64, mb = PP_INF64;
                for (int u = n - kprev; u < n; ++u)
                    for (int v = n; v < n + k; ++v) {
                        long long x = a.bw[(size_t)o[u] * D + o[v]], y = a.bw[(size_t)o[v] * D + o[u]];
                        mf = x < mf ? x : mf;
                        mb = y < mb ? y : mb;
                    }
                cf = ceil_div64(a.actf[e0 - 1], (long long)kprev * k * mf);
                cb = ceil_div64(a.actb[e0 - 1], (long long)kprev * k * mb);
            }
            e0 = e;
            n += k;
            kprev = k;
        }
        A[s] = As;
        amax = As > amax ? As : amax;
        long long w = F + Bk > cf + cb ? F + Bk : cf + cb;
        worst = w > worst ? w : worst;
        const int r = 2 * s + 1;
        if (s == S - 1) {
            dur[R] = F + Bk;
        } else {
            dur[r] = F;
            dur[2 * R - r] = Bk;
        }
        if (s) {
            dur[r - 1] = cf;
            dur[2 * R - (r - 1)] = cb;
        }
    }
    dur[0] = 0;
    if (ok) {
        fault |= overflow_fault(worst, M, S);
        if (amax >= PP_CAP62 / 2) fault |= PP_FAULT_OVERFLOW;
    }
    // the later of the last backward block on stage 0 and the end of every AllReduce
    auto finish = [&](auto &fin) {
        long long T = (long long)fin[J];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const int jb = s == S - 1 ? R : 2 * R - (2 * s + 1);
            const long long t = (long long)fin[jb] + A[s];
            T = (A[s] > 0 && t > T) ? t : T;
        }
        return T;
    };
    const bool narrow = !ok || fault || worst <= (long long)0x7fffffff / ((long long)M + 4 * S - 4);
    long long T;
    if (__all(narrow)) T = sweep_regs<S, int>(dur, M, finish);
    else T = sweep_regs<S, long long>(dur, M, finish);
    if (live) {
        if (fault) pp_raise(a.status, fault);
        a.T_out[c * a.t_stride + a.t_off] = (none || fault) ? PP_INF64 : T;
    }
}

// ---------------------------------------------------------------- LDS columns, any S

// True if no finish time of any candidate of the launch can reach 2^31 for any of its
// microbatch counts (Lemma 1's bound with the largest time of the tables); the same for every
// lane of every wave.  False without a header.
__device__ __forceinline__ bool launch_is_narrow(const mk_args &a) {
    if (!a.hdr) return false;
    unsigned long long vmax = 0;
    for (int b = 0; b < PP_PACK_BLOCKS; ++b) vmax = a.hdr->pmax[b] > vmax ? a.hdr->pmax[b] : vmax;
    int mmax = 1;
    for (int q = 0; q < a.nM; ++q) mmax = a.Ms[q] > mmax ? a.Ms[q] : mmax;
    return vmax <= 0x7fffffffull / (unsigned long long)(mmax + 4 * a.S - 4);
}

// Without a header the same question per block of 64 candidates, from the largest per-resource
// time of each of them (`worst` as gather_durations reports it; ok = this lane's candidates fit,
// dead and faulty ones count as fitting): both kernels evaluate this on the same values, so
// exactly one of them schedules the block.
__device__ __forceinline__ bool fits_narrow(const mk_args &a, long long worst) {
    int mmax = 1;
    for (int q = 0; q < a.nM; ++q) mmax = a.Ms[q] > mmax ? a.Ms[q] : mmax;
    return worst <= (long long)(0x7fffffffull / (unsigned long long)(mmax + 4 * a.S - 4));
}

// 16 < S <= 32 with 32-bit times: the 4S-3 finish times of a lane in registers (blocks
// unrolled, each update selected by a per-lane test of the sweep's window), the durations in
// the lane's LDS column.  Runs only if the whole launch is narrow; k_makespan_lds, launched
// with it, runs otherwise.
template <int S>
__global__ __launch_bounds__(64) void k_makespan_mid(mk_args a) {
    constexpr int R = 2 * S - 1, J = 2 * R - 1;
    extern __shared__ int smi[];
    if (!a.by_block && !launch_is_narrow(a)) return;
    const int lane = threadIdx.x;
    int *dur = smi + lane;  // [J][64]
    const long long c = (long long)blockIdx.x * 64 + lane;
    const bool live = c < a.N;
    long long worst;
    const int fault = gather_durations<S>(a, c, live, worst,
                                          [&](int j, long long d) { dur[(j - 1) * 64] = (int)d; });
    // (by block: this kernel takes the block iff all of its 64 candidates fit 32 bits)
    if (a.by_block && !__all(!live || fault || fits_narrow(a, worst))) return;
    for (int q = 0; q < a.nM; ++q) {
        const int M = a.Ms[q];
        const int fq = (live && !fault) ? overflow_fault(worst, M, S) : fault;
        int fin[J + 1];
#pragma unroll
        for (int j = 0; j <= J; ++j) fin[j] = 0;
        const int sweeps = M + 2 * R - 2;
        const unsigned width = (unsigned)(M - 1);
        for (int t = 1; t <= sweeps; ++t) {
            const int jlo_s = t - M + 1;  // the sweep's window is blocks jlo_s .. t
            int jlo = jlo_s;
            asm volatile("" : "+v"(jlo));
            const int finR_prev = fin[R];
            // groups of eight blocks; one that lies wholly outside the window is jumped over
            // (while the pipeline fills and drains that is about half of them)
#pragma unroll
            for (int jb = R; jb >= 1; jb -= 8) {
                const int ja = jb - 7 > 1 ? jb - 7 : 1;
                if (jb < jlo_s || ja > t) continue;
#pragma unroll
                for (int j = jb; j >= ja; --j) {
                    int idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
                    int ready = j > 1 ? fin[j - 1] : 0;
                    int nv = (idle > ready ? idle : ready) + dur[(j - 1) * 64];
                    fin[j] = (unsigned)(j - jlo) <= width ? nv : fin[j];
                }
            }
#pragma unroll
            for (int jb = J; jb >= R + 1; jb -= 8) {
                const int ja = jb - 7 > R + 1 ? jb - 7 : R + 1;
                if (jb < jlo_s || ja > t) continue;
#pragma unroll
                for (int j = jb; j >= ja; --j) {
                    int idle = fin[j] > fin[2 * R - j] ? fin[j] : fin[2 * R - j];
                    int ready = j == R + 1 ? finR_prev : fin[j - 1];
                    int nv = (idle > ready ? idle : ready) + dur[(j - 1) * 64];
                    fin[j] = (unsigned)(j - jlo) <= width ? nv : fin[j];
                }
            }
        }
        emit(a, q, c, live, fq, (long long)fin[J], blockIdx.x, gridDim.x, a.t_off);
    }
}

// blockDim.x = lanes in use (64, or fewer when 2 * (4S-3) rows of 64 int64 would not fit in
// 64 KiB of LDS); the lane's state lives in its own column [row][lane]: no bank conflicts, no
// barriers.
__global__ __launch_bounds__(64) void k_makespan_lds(mk_args a) {
    extern __shared__ long long sm[];
    const int lane = threadIdx.x, W = blockDim.x;
    const int S = a.S;
    if (S > 16 && S <= 32 && !a.by_block && launch_is_narrow(a)) return;  // k_makespan_mid does this launch
    if (a.by_block) {
        // k_makespan_mid takes the block of 64 candidates this workgroup's W lie in iff all 64
        // fit 32 bits: the same test here, every lane looking at 64 / W of them
        const long long c0 = ((long long)blockIdx.x * W / 64) * 64;
        bool ok = true;
        for (int i = lane; i < 64; i += W) {
            const long long cc = c0 + i;
            const bool lv = cc < a.N;
            long long w2;
            const int f2 = gather_durations<0>(a, cc, lv, w2, [](int, long long) {});
            ok = ok && (!lv || f2 || fits_narrow(a, w2));
        }
        if (__all(ok)) return;
    }
    const int R = 2 * S - 1, J = 2 * R - 1;
    // rows 0..J-1: duration of block j = row+1; rows J..2J-1: its latest finish time
    long long *dur = sm + lane;
    long long *fin = sm + (size_t)J * W + lane;
    const long long c = (long long)blockIdx.x * W + lane;
    const bool live = c < a.N;
    long long worst;
    const int fault = gather_durations<0>(a, c, live, worst,
                                          [&](int j, long long d) { dur[(size_t)(j - 1) * W] = d; });
  for (int q = 0; q < a.nM; ++q) {
    const int M = a.Ms[q];
    const int fq = (live && !fault) ? overflow_fault(worst, M, S) : fault;
    for (int j = 1; j <= J; ++j) fin[(size_t)(j - 1) * W] = 0;

    const int sweeps = M + 2 * R - 2;
    for (int t = 1; t <= sweeps; ++t) {
        const int jlo = max(1, t - M + 1), jhi = min(J, t);
        const long long finR_prev = fin[(size_t)(R - 1) * W];
        for (int j = min(jhi, R); j >= jlo; --j) {
            long long idle = max(fin[(size_t)(j - 1) * W], fin[(size_t)((2 * R - j) - 1) * W]);
            long long ready = j > 1 ? fin[(size_t)((j - 1) - 1) * W] : 0;
            fin[(size_t)(j - 1) * W] = max(idle, ready) + dur[(size_t)(j - 1) * W];
        }
        for (int j = jhi; j >= max(jlo, R + 1); --j) {
            long long idle = max(fin[(size_t)(j - 1) * W], fin[(size_t)((2 * R - j) - 1) * W]);
            long long ready = j == R + 1 ? finR_prev : fin[(size_t)((j - 1) - 1) * W];
            fin[(size_t)(j - 1) * W] = max(idle, ready) + dur[(size_t)(j - 1) * W];
        }
    }
    // with fewer than 64 lanes the arg-min would need another reduction; the host only asks
    // for it when W == 64
    emit(a, q, c, live, fq, fin[(size_t)(J - 1) * W], blockIdx.x, gridDim.x, a.t_off);
  }
}

static long long regs_waves(long long N) { return (N + 63) / 64; }

// S = 0: the kernel for all S <= 8 (a.S, or every stage count 1..a.S if a.all_xi is set).
template <int S>
static int launch_regs(const mk_args &a, hipStream_t st) {
    unsigned grid = (unsigned)regs_waves(a.N);
    const int nw = a.nM < MK_REGS_WAVES ? a.nM : MK_REGS_WAVES;
    const size_t lds = nw > 1 ? (size_t)(4 * (S ? S : a.S) - 3 + 1 + nw) * 64 * 8 : 0;
    mk_args b = a;
    // wave slots in descending order of the microbatch count (stable: equal counts keep theirs)
    for (int i = 0; i < PP_MAX_M_LIST; ++i) b.order[i] = (unsigned char)i;
    for (int i = 1; i < a.nM; ++i)
        for (int k = i; k > 0 && a.Ms[b.order[k]] > a.Ms[b.order[k - 1]]; --k) {
            unsigned char t = b.order[k]; b.order[k] = b.order[k - 1]; b.order[k - 1] = t;
        }
    // A launch of a few hundred workgroups is bound by the SIMD that gets the most work, and
    // the waves' work differs by the microbatch count.  The waves of a workgroup go to the four
    // SIMDs of its compute unit in cyclic order (recorded hardware ids), but where the next
    // workgroup starts varies, so with one group of four waves per workgroup two or three of
    // the longest waves often meet on one SIMD.  With four different counts the workgroup
    // therefore holds three groups (12 waves, 192 candidates) whose slot orders are permuted so
    // that the three waves a SIMD gets from it (w, w + 4, w + 8) add up to about the same
    // number of sweeps on every SIMD, wherever the workgroup lands.
    b.groups = 1;
    b.slot_perm = 0xE4E4E4;  // identity three times
    unsigned gridx = grid;
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        cus = 256;
    // (with no more groups than compute units every wave has a SIMD of its own anyway)
    if (S == 0 && nw == 4 && a.nM == 4 && !a.all_xi && !a.rlist && grid > (unsigned)cus) {
        long long wt[4];
        for (int i = 0; i < 4; ++i) wt[i] = a.Ms[b.order[i]];
        int perms[24][4], np = 0;
        for (int p0 = 0; p0 < 4; ++p0) for (int p1 = 0; p1 < 4; ++p1) for (int p2 = 0; p2 < 4; ++p2) {
            const int p3 = 6 - p0 - p1 - p2;
            if (p0 == p1 || p0 == p2 || p1 == p2 || p3 < 0 || p3 > 3 || p3 == p0 || p3 == p1 || p3 == p2) continue;
            perms[np][0] = p0; perms[np][1] = p1; perms[np][2] = p2; perms[np][3] = p3; ++np;
        }
        long long best = -1;
        for (int i1 = 0; i1 < np; ++i1) for (int i2 = 0; i2 < np; ++i2) {
            long long m = 0;
            for (int sd = 0; sd < 4; ++sd) {
                const long long sum = wt[sd] + wt[perms[i1][sd]] + wt[perms[i2][sd]];
                m = sum > m ? sum : m;
            }
            if (best < 0 || m < best) {
                best = m;
                unsigned bits = 0xE4;
                for (int w = 0; w < 4; ++w) bits |= (unsigned)perms[i1][w] << (2 * (4 + w)) | (unsigned)perms[i2][w] << (2 * (8 + w));
                b.slot_perm = bits;
            }
        }
        b.groups = MK_REGS_GROUPS;
        gridx = (grid + MK_REGS_GROUPS - 1) / MK_REGS_GROUPS;
    }
    size_t lds_all = lds * b.groups;
    if (b.fuse) {
        const size_t need = mk_fuse_lds_bytes(a.L, a.D, a.S, nw, b.groups);
        lds_all = need > lds_all ? need : lds_all;
    }
    if constexpr (S == 0) {
        if (a.rlist)
            hipLaunchKernelGGL(k_makespan_regs8_listed, dim3(grid, (a.nM + nw - 1) / nw, a.all_xi ? a.S : 1),
                               dim3(64 * nw), lds, st, b);
        else if (a.all_xi && a.share[a.S > 2 ? a.S - 2 : 0] > 1)
            hipLaunchKernelGGL(k_makespan_regs8_shared, dim3(grid, (a.nM + nw - 1) / nw, a.S),
                               dim3(64 * nw), lds, st, b);
        else
            hipLaunchKernelGGL(k_makespan_regs8, dim3(gridx, (a.nM + nw - 1) / nw, a.all_xi ? a.S : 1),
                               dim3(64 * nw * b.groups), lds_all, st, b);
    }
    else
        hipLaunchKernelGGL(k_makespan_regs<S>, dim3(grid, (a.nM + nw - 1) / nw), dim3(64 * nw), lds, st, b);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

template <int S>
static int launch_mid(const mk_args &a, hipStream_t st) {
    unsigned grid = (unsigned)((a.N + 63) / 64);
    hipLaunchKernelGGL(k_makespan_mid<S>, dim3(grid), dim3(64), (size_t)(4 * S - 3) * 64 * 4, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

static void plain_layout(mk_args &a, int S) {
    a.ord_stride = S; a.bnd_stride = S; a.bnd_off = 0; a.t_stride = 1; a.t_off = 0; a.search = 0;
    a.reps = NULL; a.PA = a.actf = a.actb = a.bw = a.W = NULL; a.rout = NULL;
    a.variant = 0;
    a.hdr = NULL;
}

// Lanes per workgroup of the LDS kernel: as many as keep 2J rows of int64 within 64 KiB.
static int lds_lanes(int S) {
    const int J = 4 * S - 3;
    int W = 64;
    while ((size_t)2 * J * W * 8 > 64 * 1024) W >>= 1;
    return W;
}

// Register kernel for a.S <= 16, LDS kernel beyond.  With a.part set the LDS kernel must run
// full waves (lds_lanes(a.S) == 64).
static int launch_makespan(const mk_args &a, hipStream_t st) {
    if (a.S <= 8) return launch_regs<0>(a, st);
    switch (a.S) {
#define CASE(n) case n: return launch_regs<n>(a, st);
        CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
    }
    const int W = lds_lanes(a.S);
    mk_args b = a;
    b.by_block = 0;
    if (!a.hdr && !a.part && a.S <= 32) {
        // no workspace header to tell whether the times fit 32 bits: both kernels are enqueued
        // and every block of 64 candidates goes to one of them (W divides 64)
        b.by_block = 1;
        int rc = PP_ERR_INVALID_ARG;
        switch (a.S) {
#define CASE(n) case n: rc = launch_mid<n>(b, st); break;
            CASE(17) CASE(18) CASE(19) CASE(20) CASE(21) CASE(22) CASE(23) CASE(24)
            CASE(25) CASE(26) CASE(27) CASE(28) CASE(29) CASE(30) CASE(31) CASE(32)
#undef CASE
        }
        if (rc) return rc;
    }
    if (a.hdr && a.S <= 32 && (W == 64 || !a.part)) {
        // both kernels are enqueued; which one works depends on the data (see launch_is_narrow)
        int rc = PP_ERR_INVALID_ARG;
        switch (a.S) {
#define CASE(n) case n: rc = launch_mid<n>(a, st); break;
            CASE(17) CASE(18) CASE(19) CASE(20) CASE(21) CASE(22) CASE(23) CASE(24)
            CASE(25) CASE(26) CASE(27) CASE(28) CASE(29) CASE(30) CASE(31) CASE(32)
#undef CASE
        }
        if (rc) return rc;
    }
    const size_t lds = (size_t)2 * (4 * a.S - 3) * W * 8;
    unsigned grid = (unsigned)((a.N + W - 1) / W);
    hipLaunchKernelGGL(k_makespan_lds, dim3(grid), dim3(W), lds, st, b);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

// The kernels that can schedule a list of representatives instead of all candidates.
bool pp_makespan_takes_list(int S) { return S >= 1 && S <= 16; }

// The makespan kernel can build the plans itself (closed form, tables staged in LDS) for 2..8
// stages when its tables fit beside the exchange area of the largest workgroup it may use.
bool pp_makespan_can_fuse(int L, int D, int S) {
    return S >= 2 && S <= 8 && D <= 32 &&
           mk_fuse_lds_bytes(L, D, S, MK_REGS_WAVES, MK_REGS_GROUPS) <= 64 * 1024;
}

int pp_launch_makespan(int L, int D, int S, int64_t N, int nM, const int *Ms, const int64_t *PF,
                       const int64_t *PB, const int64_t *XF, const int64_t *XB,
                       const int32_t *orderings, const int32_t *bounds, int64_t *T_out,
                       int64_t *T_scratch, int32_t *status, const int64_t *C, void *part,
                       pp_result *out, const pp_ws_header *hdr, const pp_fuse_info *fuse,
                       const int32_t *rlist, hipStream_t st) {
    if (rlist && (!pp_makespan_takes_list(S) || !hdr || !part)) return PP_ERR_INVALID_ARG;
    mk_args a = {};
    a.rlist = rlist;
    a.L = L; a.D = D; a.S = S; a.N = N;
    a.nM = nM;
    for (int q = 0; q < PP_MAX_M_LIST; ++q) a.Ms[q] = q < nM ? Ms[q] : 1;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.orderings = orderings; a.bounds = bounds;
    plain_layout(a, S);
    a.T_out = (long long *)T_out; a.status = status;
    a.part = (tc_pair *)part; a.C = (const long long *)C; a.out = out;
    a.hdr = hdr;
    if (fuse && hdr && !rlist && pp_makespan_can_fuse(L, D, S)) {
        a.fuse = 1;
        a.fuse_mmax = fuse->mmax;
        a.fuse_validate = fuse->validate;
        a.bfl = (const long long *)fuse->bfl;
        a.C_w = (long long *)fuse->C;
        a.bounds_w = fuse->bounds;
    }
    if (S > 16 && lds_lanes(S) != 64 && part) {
        // narrow workgroups: per microbatch count, T goes to memory and a separate pass finds
        // the minimum
        for (int q = 0; q < nM; ++q) {
            mk_args b = a;
            b.nM = 1; b.Ms[0] = Ms[q];
            b.part = NULL; b.C = NULL; b.out = NULL;
            b.T_out = T_out ? (long long *)T_out + (long long)q * N : (long long *)T_scratch;
            if (!b.T_out) return PP_ERR_INVALID_ARG;
            int rc = launch_makespan(b, st);
            if (rc) return rc;
            rc = pp_launch_argmin(D, S, N, (const int64_t *)b.T_out, C, bounds, orderings, part,
                                  out + q, st);
            if (rc) return rc;
        }
        return PP_OK;
    }
    int rc = launch_makespan(a, st);
    if (rc || !part) return rc;
    // one partial per wave of 64 candidates and microbatch count
    return launch_pick(a, nM, S <= 16 ? regs_waves(N) : (N + 63) / 64, st);
}

// ---------------------------------------------------------------- stand-alone arg-min

// Each wave reduces a strided share of T (blockIdx.y selects the microbatch count) to a partial
// for k_pick.
__global__ __launch_bounds__(64) void k_argmin(mk_args a) {
    const int lane = threadIdx.x, q = blockIdx.y;
    const long long *T = a.T_out + (long long)q * a.N;
    tc_pair v = {PP_INF64, INT64_MAX};
    if (a.rlist && a.hdr->share_active) {
        // only the rows of the representatives hold values: entry (r, x) of the list is entry
        // rep(r) * w + x of T (w entries per candidate: the stage counts of the search)
        const long long w = a.search ? a.search : 1, todo = (long long)a.hdr->share_nreps * w;
        for (long long i = (long long)blockIdx.x * 64 + lane; i < todo; i += (long long)gridDim.x * 64) {
            const long long r = i / w, c = pp_share_at(a.hdr, a.rlist, a.N / w, r) * w + (i - r * w);
            tc_pair o = {T[c], c};
            v = tc_min(v, o);
        }
    } else {
        for (long long c = (long long)blockIdx.x * 64 + lane; c < a.N; c += (long long)gridDim.x * 64) {
            tc_pair o = {T[c], c};
            v = tc_min(v, o);
        }
    }
    // emit() reduces over the wave: hand it this lane's minimum as if it were the lane's own
    // candidate; T_out must not be rewritten
    mk_args b = a;
    b.T_out = NULL;
    emit(b, q, v.c, v.c != INT64_MAX, 0, v.T, blockIdx.x, gridDim.x, b.t_off);
}

int pp_launch_argmin(int D, int S, int64_t N, const int64_t *T, const int64_t *C,
                     const int32_t *bounds, const int32_t *orderings, void *part,
                     pp_result *out, hipStream_t st) {
    mk_args a = {};
    a.L = 0; a.D = D; a.S = S; a.N = N;
    a.nM = 1;
    for (int q = 0; q < PP_MAX_M_LIST; ++q) a.Ms[q] = 1;
    a.PF = a.PB = a.XF = a.XB = NULL;
    a.orderings = orderings; a.bounds = bounds;
    plain_layout(a, S);
    a.T_out = (long long *)T; a.status = NULL;
    a.part = (tc_pair *)part; a.C = (const long long *)C; a.out = out;
    long long waves = (N + 63) / 64;
    if (waves > 1024) waves = 1024;
    hipLaunchKernelGGL(k_argmin, dim3((unsigned)waves), dim3(64), 0, st, a);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return launch_pick(a, 1, waves, st);
}

// ---------------------------------------------------------------- stage-count search

int pp_launch_makespan_stages(int L, int D, int S, int64_t N, int nM, const int *Ms,
                              const int64_t *PF, const int64_t *PB, const int64_t *XF,
                              const int64_t *XB, const int32_t *orderings, const int32_t *bounds,
                              const int64_t *C, int64_t *T_st, int32_t *status, void *part,
                              pp_result *out, const pp_ws_header *hdr, int lex,
                              const int32_t *rlist, hipStream_t st) {
    if (rlist && (!pp_makespan_takes_list(S) || !hdr)) return PP_ERR_INVALID_ARG;
    mk_args a = {};
    a.rlist = rlist;
    a.L = L; a.D = D; a.N = N; a.nM = nM;
    for (int q = 0; q < PP_MAX_M_LIST; ++q) a.Ms[q] = q < nM ? Ms[q] : 1;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.orderings = orderings; a.bounds = bounds;
    a.T_out = (long long *)T_st; a.status = status;
    a.part = NULL; a.C = NULL; a.out = NULL;
    a.ord_stride = S; a.bnd_stride = (long long)S * (S + 1) / 2; a.t_stride = S; a.search = 0;
    a.reps = NULL; a.PA = a.actf = a.actb = a.bw = a.W = NULL; a.rout = NULL;
    a.variant = 0; a.hdr = hdr;
    if (S <= 8) {
        // the schedules of xi stages on the first xi devices, every xi in one launch
        a.S = S; a.all_xi = 1;
        a.bnd_off = 0; a.t_off = 0;
        for (int xi = 0; xi <= 8; ++xi) {
            long long fct = 1;
            if (lex && xi >= 1) for (int i = 2; i <= D - xi; ++i) fct *= i;  // D = S <= 8 here
            // (long blocks are not worth it: few waves would write thousands of entries each,
            // and the plans with few stages are the cheap ones anyway)
            a.share[xi] = fct <= 32 ? fct : 1;
        }
        int rc = launch_makespan(a, st);
        if (rc) return rc;
        a.all_xi = 0;
    } else {
        // one launch per stage count
        for (int xi = 1; xi <= S; ++xi) {
            a.S = xi;
            a.bnd_off = xi * (xi - 1) / 2;
            a.t_off = xi - 1;
            int rc = launch_makespan(a, st);
            if (rc) return rc;
        }
    }
    // smallest T over all (candidate, stage count) pairs, lowest c*S + xi-1 on ties
    mk_args m = a;
    m.S = S; m.N = N * S; m.search = S;
    m.part = (tc_pair *)part; m.C = (const long long *)C; m.out = out;
    long long waves = (m.N + 63) / 64;
    if (waves > 1024) waves = 1024;
    hipLaunchKernelGGL(k_argmin, dim3((unsigned)waves, nM), dim3(64), 0, st, m);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return launch_pick(m, nM, waves, st);
}

// ---------------------------------------------------------------- replicated stages: launch

template <int S>
static int launch_rep(const mk_args &a, hipStream_t st) {
    unsigned grid = (unsigned)((a.N + 63) / 64);
    hipLaunchKernelGGL(k_rep_makespan<S>, dim3(grid), dim3(64), 0, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}

int pp_launch_rep_makespan(int L, int D, int64_t N, int M, const int64_t *PF, const int64_t *PB,
                           const int64_t *PA, const int64_t *actf, const int64_t *actb,
                           const int64_t *bw, const int32_t *orderings, const int32_t *bounds,
                           const int32_t *reps, const int64_t *W, int64_t *T_out, int32_t *status,
                           void *part, pp_rep_result *out, hipStream_t st) {
    if (D > 16) return PP_ERR_INVALID_ARG;
    mk_args a = {};
    a.L = L; a.D = D; a.N = N; a.nM = 1;
    for (int q = 0; q < PP_MAX_M_LIST; ++q) a.Ms[q] = M;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = a.XB = NULL;
    a.PA = (const long long *)PA; a.actf = (const long long *)actf; a.actb = (const long long *)actb;
    a.bw = (const long long *)bw; a.W = (const long long *)W;
    a.orderings = orderings; a.bounds = bounds; a.reps = reps;
    a.T_out = (long long *)T_out; a.status = status;
    a.part = NULL; a.C = NULL; a.out = NULL; a.rout = NULL;
    a.ord_stride = D; a.bnd_stride = (long long)D * (D + 1) / 2; a.t_stride = D; a.search = 0;
    for (int xi = 1; xi <= D; ++xi) {
        a.S = xi;
        a.bnd_off = xi * (xi - 1) / 2;
        a.t_off = xi - 1;
        int rc = PP_ERR_INVALID_ARG;
        switch (xi) {
#define CASE(n) case n: rc = launch_rep<n>(a, st); break;
            CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
            CASE(9) CASE(10) CASE(11) CASE(12) CASE(13) CASE(14) CASE(15) CASE(16)
#undef CASE
        }
        if (rc) return rc;
    }
    // smallest T over all (candidate, stage count) pairs, lowest c*D + xi-1 on ties
    mk_args m = a;
    m.S = D; m.N = N * D; m.search = D;
    m.part = (tc_pair *)part; m.C = (const long long *)W; m.rout = out;
    long long waves = (m.N + 63) / 64;
    if (waves > 1024) waves = 1024;
    hipLaunchKernelGGL(k_argmin, dim3((unsigned)waves, 1), dim3(64), 0, st, m);
    if (hipGetLastError() != hipSuccess) return PP_ERR_HIP;
    return launch_pick(m, 1, waves, st);
}

// ---------------------------------------------------------------- schedule variants

// Comparison schedules with the timing rule of Alg. 1's scheduling phase, any S, one lane per
// candidate, the lane's state in its own LDS column (rows [row][lane]).
//   PP_SCHED_DUPLEX: the sweeps of the PE scheduler, but the forward and backward transfers of
//     a stage pair have a channel each, so a channel block waits only for its own previous item.
//   PP_SCHED_GPIPE: every stage and channel serves all forward items before any backward item
//     (Sec. II: "all FP before starting any BP"), microbatches in order.  With that order the
//     resources form a flow shop: the forward wave is busy[r] = max(busy[r], busy of the same
//     microbatch on r-1) + forward time, resources 1..R, microbatch by microbatch; the backward
//     wave the same in the other direction, each resource continuing from the end of its last
//     forward item.  The last stage's forward and backward passes are separate items here.
//   PP_SCHED_ADDITIVE: the sweeps of the PE scheduler over the 2S-1 stage blocks alone, each
//     with the transfers over the stage's inbound link added to its duration.
//   PP_SCHED_FIFO: Alg. 1 with channels that serve by readiness instead of by list (only
//     computation blocks enter the lists U_s in the listing): an event simulation.
__global__ __launch_bounds__(64) void k_makespan_variant(mk_args a) {
    extern __shared__ long long sm[];
    const int lane = threadIdx.x, W = blockDim.x;
    const int S = a.S, M = a.Ms[0];
    const int R = 2 * S - 1, J = 2 * R - 1;
    long long *dur = sm + lane;                    // rows 0..J-1: duration of block j = row + 1
    long long *fin = sm + (size_t)J * W + lane;    // rows J..2J-1: finish times / busy-until times
    const long long c = (long long)blockIdx.x * W + lane;
    const bool live = c < a.N;
    long long worst, lastF = 0, lastB = 0;
    const int fault0 = gather_durations<0>(a, c, live, worst,
                                           [&](int j, long long d) { dur[(size_t)(j - 1) * W] = d; },
                                           [&](long long F, long long B) { lastF = F; lastB = B; });
    const int fault = (live && !fault0) ? overflow_fault(worst, M, S) : fault0;
    for (int j = 1; j <= J; ++j) fin[(size_t)(j - 1) * W] = 0;
    long long T;
    if (a.variant == PP_SCHED_GPIPE) {
        // busy[r] lives in fin row r-1; forward time of resource r = dur of block r (the last
        // stage's forward alone), backward time = dur of block 2R - r (the last stage's backward)
        for (int m = 0; m < M; ++m) {
            long long prev = 0;
            for (int r = 1; r <= R; ++r) {
                const long long d = r == R ? lastF : dur[(size_t)(r - 1) * W];
                long long b = fin[(size_t)(r - 1) * W];
                b = (b > prev ? b : prev) + d;
                fin[(size_t)(r - 1) * W] = b;
                prev = b;
            }
        }
        for (int m = 0; m < M; ++m) {
            long long prev = 0;
            for (int r = R; r >= 1; --r) {
                const long long d = r == R ? lastB : dur[(size_t)(2 * R - r - 1) * W];
                long long b = fin[(size_t)(r - 1) * W];
                b = (b > prev ? b : prev) + d;
                fin[(size_t)(r - 1) * W] = b;
                prev = b;
            }
        }
        T = fin[0];
    } else if (a.variant == PP_SCHED_FIFO) {
        // Event simulation, one committed item per iteration (the same in every lane): every
        // block handles the microbatches in index order, nxt[j] is block j's next one.  A
        // stage's next item is the earlier of its two blocks' heads in list order (sweep
        // m + j - 1, then block); a channel takes, of its heads whose microbatch has left the
        // preceding block, the one that left it first (equal: earlier in list order).  The item
        // with the earliest start over all resources is committed (equal: lowest resource).
        // A microbatch is in exactly one place, so one "left its last block at" time per
        // microbatch in flight is enough; the first stage's list keeps at most J in flight,
        // so they live in a ring of Q >= J slots (Q a power of two).
        int Q = 1;
        while (Q < J) Q <<= 1;
        long long *idle = fin;                              // rows J..J+R-1: resource r at r-1
        long long *ring = fin + (size_t)R * W;              // Q rows
        long long *nxt = ring + (size_t)Q * W;              // J rows: block j at j-1
        for (int r = 0; r < R; ++r) idle[(size_t)r * W] = 0;
        for (int q = 0; q < Q; ++q) ring[(size_t)q * W] = 0;
        for (int j = 0; j < J; ++j) nxt[(size_t)j * W] = 1;
        T = 0;
        for (long long left = (long long)J * M; left > 0; --left) {
            int best_r = 0, best_j = 0;
            long long best_start = 0;
            for (int r = 1; r <= R; ++r) {
                const int ja = r, jb = 2 * R - r;
                const int ma = (int)nxt[(size_t)(ja - 1) * W], mb = (int)nxt[(size_t)(jb - 1) * W];
                // head (m, j) of a block is there once block j-1 has moved past m
                const bool at_a = ma <= M && (ja == 1 || (int)nxt[(size_t)(ja - 2) * W] > ma);
                const bool at_b = jb != ja && mb <= M && (int)nxt[(size_t)(jb - 2) * W] > mb;
                const long long ra = ja == 1 ? 0 : ring[(size_t)(ma & (Q - 1)) * W];
                const long long rb = ring[(size_t)(mb & (Q - 1)) * W];
                int j = 0;
                if (r & 1) {
                    const bool has_a = ma <= M, has_b = jb != ja && mb <= M;
                    if (has_a && (!has_b || ma + ja <= mb + jb)) j = at_a ? ja : 0;
                    else if (has_b) j = at_b ? jb : 0;
                } else {
                    const bool a_first = ra < rb || (ra == rb && ma + ja <= mb + jb);
                    if (at_a && (!at_b || a_first)) j = ja;
                    else if (at_b) j = jb;
                }
                const long long ready = j == ja ? ra : rb;
                const long long busy = idle[(size_t)(r - 1) * W];
                const long long start = ready > busy ? ready : busy;
                if (j && (!best_r || start < best_start)) { best_r = r; best_j = j; best_start = start; }
            }
            // (there always is one: block 1 or the successor of a finished item)
            if (best_r) {
                const long long f = best_start + dur[(size_t)(best_j - 1) * W];
                const int m = (int)nxt[(size_t)(best_j - 1) * W];
                ring[(size_t)(m & (Q - 1)) * W] = f;
                idle[(size_t)(best_r - 1) * W] = f;
                nxt[(size_t)(best_j - 1) * W] = m + 1;
                if (best_j == J) T = f > T ? f : T;
            }
        }
    } else {
        // The PE sweeps over a list of 2Rv-1 blocks on Rv resources, block j and block 2Rv-j on
        // the same one.  DUPLEX: the standard list, but even resources are channels, whose two
        // blocks do not wait for each other.  ADDITIVE: the stage blocks only.
        int Rv = R;
        const bool pair_all = a.variant == PP_SCHED_ADDITIVE;
        if (pair_all && S > 1) {
            // stage n's forward block 2n+1 and backward block 2R-(2n+1) of the standard list
            // take in the channel blocks 2n and 2R-2n; the merged block R both of its channel's.
            // New list: forward of stage n at n+1, merged block at S, backward of stage n at
            // 2S-1-n.  Built in the finish-time rows first, then moved.
            for (int n = 0; n < S - 1; ++n) {
                const int jf = 2 * n + 1, jb = 2 * R - jf;
                long long df = dur[(size_t)(jf - 1) * W], db = dur[(size_t)(jb - 1) * W];
                if (n) { df += dur[(size_t)(jf - 2) * W]; db += dur[(size_t)jb * W]; }
                fin[(size_t)n * W] = df;
                fin[(size_t)(2 * S - 2 - n) * W] = db;
            }
            fin[(size_t)(S - 1) * W] = dur[(size_t)(R - 1) * W] + dur[(size_t)(R - 2) * W] + dur[(size_t)R * W];
            for (int j = 1; j <= 2 * S - 1; ++j) {
                dur[(size_t)(j - 1) * W] = fin[(size_t)(j - 1) * W];
                fin[(size_t)(j - 1) * W] = 0;
            }
            Rv = S;
        }
        const int Jv = 2 * Rv - 1, sweeps = M + Jv - 1;
        for (int t = 1; t <= sweeps; ++t) {
            const int jlo = max(1, t - M + 1), jhi = min(Jv, t);
            const long long finR_prev = fin[(size_t)(Rv - 1) * W];
            for (int j = min(jhi, Rv); j >= jlo; --j) {
                long long idle = fin[(size_t)(j - 1) * W];
                if (pair_all || (j & 1)) idle = max(idle, fin[(size_t)((2 * Rv - j) - 1) * W]);
                long long ready = j > 1 ? fin[(size_t)((j - 1) - 1) * W] : 0;
                fin[(size_t)(j - 1) * W] = max(idle, ready) + dur[(size_t)(j - 1) * W];
            }
            for (int j = jhi; j >= max(jlo, Rv + 1); --j) {
                long long idle = fin[(size_t)(j - 1) * W];
                if (pair_all || (j & 1)) idle = max(idle, fin[(size_t)((2 * Rv - j) - 1) * W]);
                long long ready = j == Rv + 1 ? finR_prev : fin[(size_t)((j - 1) - 1) * W];
                fin[(size_t)(j - 1) * W] = max(idle, ready) + dur[(size_t)(j - 1) * W];
            }
        }
        T = fin[(size_t)(Jv - 1) * W];
    }
    if (live) {
        if (fault) pp_raise(a.status, fault);
        a.T_out[c] = fault ? PP_INF64 : T;
    }
}

int pp_launch_makespan_variant(int variant, int L, int D, int S, int64_t N, int M, const int64_t *PF,
                               const int64_t *PB, const int64_t *XF, const int64_t *XB,
                               const int32_t *orderings, const int32_t *bounds, int64_t *T_out,
                               int32_t *status, hipStream_t st) {
    mk_args a = {};
    a.L = L; a.D = D; a.S = S; a.N = N; a.nM = 1;
    for (int q = 0; q < PP_MAX_M_LIST; ++q) a.Ms[q] = M;
    a.PF = (const long long *)PF; a.PB = (const long long *)PB;
    a.XF = (const long long *)XF; a.XB = (const long long *)XB;
    a.orderings = orderings; a.bounds = bounds;
    plain_layout(a, S);
    a.variant = variant;
    a.T_out = (long long *)T_out; a.status = status;
    a.part = NULL; a.C = NULL; a.out = NULL;
    int W = lds_lanes(S);
    const int J = 4 * S - 3, R = 2 * S - 1;
    size_t rows = (size_t)2 * J;
    if (variant == PP_SCHED_FIFO) {
        // durations, resource idle times, a power-of-two ring of J or more, next microbatches
        int Q = 1;
        while (Q < J) Q <<= 1;
        rows = (size_t)J + R + Q + J;
        W = 64;
        while (rows * W * 8 > 64 * 1024) W >>= 1;
    }
    const size_t lds = rows * W * 8;
    unsigned grid = (unsigned)((N + W - 1) / W);
    hipLaunchKernelGGL(k_makespan_variant, dim3(grid), dim3(W), lds, st, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_HIP;
}
