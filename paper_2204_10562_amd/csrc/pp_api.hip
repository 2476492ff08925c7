// Entry points of libpp that only check arguments and enqueue kernels.
#include <atomic>

#include "pp_common.h"

static bool factorial_is(int D, int64_t N) {
    int64_t f = 1;
    for (int i = 2; i <= D; ++i) {
        if (f > INT64_MAX / i) return false;
        f *= i;
    }
    return f == N;
}

int pp_check_sizes(int L, int D, int S, int64_t N, const int32_t *orderings) {
    if (L < 1 || L > PP_MAX_LAYERS || D < 1 || D > PP_MAX_DEVICES) return PP_ERR_INVALID_ARG;
    if (S < 1 || S > L || S > D || S > PP_MAX_STAGES || N < 1) return PP_ERR_INVALID_ARG;
    if (!orderings && (S != D || D > 20 || !factorial_is(D, N))) return PP_ERR_INVALID_ARG;
    return PP_OK;
}

extern "C" size_t pp_workspace_bytes(int L, int D, int S, int64_t N) {
    if (L < 1 || L > PP_MAX_LAYERS || D < 1 || D > PP_MAX_DEVICES) return 0;
    if (S < 1 || S > L || S > D || S > PP_MAX_STAGES || N < 1) return 0;
    return pp_layout(L, D, S, N).total;
}

static int check_ws(const void *ws, size_t bytes, const pp_ws_layout &lay) {
    if (!ws || ((uintptr_t)ws & 255) || bytes < lay.total) return PP_ERR_WORKSPACE;
    return PP_OK;
}

extern "C" int pp_partition_dp(int L, int D, int S, int64_t N, const int64_t *PF,
                               const int64_t *PB, const int64_t *XF, const int64_t *XB,
                               const int32_t *orderings, int64_t *C_out, int32_t *bounds_out,
                               void *workspace, size_t workspace_bytes, int32_t *status,
                               void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (!PF || !PB || !XF || !XB || !C_out || !bounds_out) return PP_ERR_INVALID_ARG;
    pp_ws_layout lay = pp_layout(L, D, S, N);
    rc = check_ws(workspace, workspace_bytes, lay);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int32_t *ord = NULL;
    rc = pp_launch_pack(L, D, S, N, PF, PB, XF, XB, orderings, workspace, lay, &ord, st);
    if (rc) return rc;
    return pp_launch_dp(L, D, S, N, PF, PB, XF, XB, orderings ? NULL : ord, orderings, 0, 0, 0, C_out,
                        bounds_out, workspace, lay, status, st);
}

extern "C" size_t pp_workspace_bytes_stages(int L, int D, int S, int64_t N, int nM) {
    if (nM < 1 || nM > PP_MAX_M_LIST || !pp_workspace_bytes(L, D, S, N)) return 0;
    return pp_layout_stages(pp_layout(L, D, S, N), S, N, nM).total;
}

extern "C" int pp_partition_dp_stages(int L, int D, int S, int64_t N, const int64_t *PF,
                                      const int64_t *PB, const int64_t *XF, const int64_t *XB,
                                      const int32_t *orderings, int64_t *C_out,
                                      int32_t *bounds_out, void *workspace,
                                      size_t workspace_bytes, int32_t *status, void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (!PF || !PB || !XF || !XB || !C_out || !bounds_out) return PP_ERR_INVALID_ARG;
    pp_ws_layout lay = pp_layout(L, D, S, N);
    rc = check_ws(workspace, workspace_bytes, lay);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int32_t *ord = NULL;
    rc = pp_launch_pack(L, D, S, N, PF, PB, XF, XB, orderings, workspace, lay, &ord, st);
    if (rc) return rc;
    return pp_launch_dp(L, D, S, N, PF, PB, XF, XB, orderings ? NULL : ord, orderings, 1, 0, 0, C_out,
                        bounds_out, workspace, lay, status, st);
}

extern "C" int pp_best_plan_stages(int L, int D, int S, int64_t N, int nM, const int32_t *M_list,
                                   const int64_t *PF, const int64_t *PB, const int64_t *XF,
                                   const int64_t *XB, const int32_t *orderings, pp_result *out,
                                   int64_t *T_all, int64_t *C_all, void *workspace,
                                   size_t workspace_bytes, int32_t *status, void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (nM < 1 || nM > PP_MAX_M_LIST || !M_list || !PF || !PB || !XF || !XB || !out)
        return PP_ERR_INVALID_ARG;
    for (int q = 0; q < nM; ++q)
        if (M_list[q] < 1) return PP_ERR_INVALID_ARG;
    pp_ws_layout lay = pp_layout(L, D, S, N);
    pp_stage_layout sl = pp_layout_stages(lay, S, N, nM);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sl.total)
        return PP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)workspace;
    int64_t *C = C_all ? C_all : (int64_t *)(base + sl.C);
    int64_t *T = T_all ? T_all : (int64_t *)(base + sl.T);
    int32_t *bounds = (int32_t *)(base + sl.bounds);
    const int32_t *ord = NULL;
    rc = pp_launch_pack(L, D, S, N, PF, PB, XF, XB, orderings, workspace, lay, &ord, st);
    if (rc) return rc;
    // (where candidates share their DP the plans of the representatives are scheduled and
    // compared, and the others get T and C only if the caller wants the arrays)
    const bool listed = lay.sh_table != 0 && pp_makespan_takes_list(S);
    rc = pp_launch_dp(L, D, S, N, PF, PB, XF, XB, orderings ? NULL : ord, orderings, 1, 0, listed, C,
                      bounds, workspace, lay, status, st);
    if (rc) return rc;
    rc = pp_launch_makespan_stages(L, D, S, N, nM, M_list, PF, PB, XF, XB, ord, bounds, C, T,
                                   status, base + sl.part, out, (const pp_ws_header *)(base + lay.hdr),
                                   orderings == NULL, listed ? (const int32_t *)(base + lay.sh_reps) : NULL,
                                   st);
    if (rc || !listed || (!T_all && !C_all)) return rc;
    return pp_launch_share_scatter(N, C_all ? S : 0, 0, T_all ? nM : 0, S, C_all, NULL, T_all, workspace,
                                   lay, st);
}

extern "C" int pp_schedule_makespan(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                                    const int64_t *PB, const int64_t *XF, const int64_t *XB,
                                    const int32_t *orderings, const int32_t *bounds,
                                    int64_t *T_out, int32_t *status, void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (M < 1 || !PF || !PB || !XF || !XB || !bounds || !T_out) return PP_ERR_INVALID_ARG;
    return pp_launch_makespan(L, D, S, N, 1, &M, PF, PB, XF, XB, orderings, bounds, T_out, NULL,
                              status, NULL, NULL, NULL, NULL, NULL, NULL, (hipStream_t)stream);
}

extern "C" int pp_schedule_makespan_multi(int L, int D, int S, int64_t N, int nM,
                                          const int32_t *M_list, const int64_t *PF,
                                          const int64_t *PB, const int64_t *XF, const int64_t *XB,
                                          const int32_t *orderings, const int32_t *bounds,
                                          int64_t *T_out, int32_t *status, void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (nM < 1 || nM > PP_MAX_M_LIST || !M_list || !PF || !PB || !XF || !XB || !bounds || !T_out)
        return PP_ERR_INVALID_ARG;
    for (int q = 0; q < nM; ++q)
        if (M_list[q] < 1) return PP_ERR_INVALID_ARG;
    return pp_launch_makespan(L, D, S, N, nM, M_list, PF, PB, XF, XB, orderings, bounds, T_out, NULL,
                              status, NULL, NULL, NULL, NULL, NULL, NULL, (hipStream_t)stream);
}

extern "C" int pp_schedule_makespan_variant(int variant, int L, int D, int S, int64_t N, int M,
                                            const int64_t *PF, const int64_t *PB, const int64_t *XF,
                                            const int64_t *XB, const int32_t *orderings,
                                            const int32_t *bounds, int64_t *T_out, int32_t *status,
                                            void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (M < 1 || !PF || !PB || !XF || !XB || !bounds || !T_out) return PP_ERR_INVALID_ARG;
    if (variant == PP_SCHED_PE)
        return pp_launch_makespan(L, D, S, N, 1, &M, PF, PB, XF, XB, orderings, bounds, T_out, NULL,
                                  status, NULL, NULL, NULL, NULL, NULL, NULL, (hipStream_t)stream);
    if (variant != PP_SCHED_DUPLEX && variant != PP_SCHED_GPIPE && variant != PP_SCHED_ADDITIVE &&
        variant != PP_SCHED_FIFO)
        return PP_ERR_INVALID_ARG;
    return pp_launch_makespan_variant(variant, L, D, S, N, M, PF, PB, XF, XB, orderings, bounds, T_out,
                                      status, (hipStream_t)stream);
}

extern "C" int pp_best_plan_multi(int L, int D, int S, int64_t N, int nM, const int32_t *M_list,
                                  const int64_t *PF, const int64_t *PB, const int64_t *XF,
                                  const int64_t *XB, const int32_t *orderings, pp_result *out,
                                  int64_t *T_all, int64_t *C_all, void *workspace,
                                  size_t workspace_bytes, int32_t *status, void *stream) {
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (nM < 1 || nM > PP_MAX_M_LIST || !M_list || !PF || !PB || !XF || !XB || !out)
        return PP_ERR_INVALID_ARG;
    for (int q = 0; q < nM; ++q)
        if (M_list[q] < 1) return PP_ERR_INVALID_ARG;
    pp_ws_layout lay = pp_layout(L, D, S, N);
    rc = check_ws(workspace, workspace_bytes, lay);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)workspace;
    int64_t *C = C_all ? C_all : (int64_t *)(base + lay.C);
    int32_t *bounds = (int32_t *)(base + lay.bounds);
    const int32_t *ord = NULL;
    rc = pp_launch_pack(L, D, S, N, PF, PB, XF, XB, orderings, workspace, lay, &ord, st);
    if (rc) return rc;
    // When the closed form of the DP applies, the makespan kernel builds the plans itself from
    // tables in LDS (one launch fewer that does work, and no trip to memory for the plans).
    // Both kernels decide on the device, from the same header, whether that is the case.
    pp_fuse_info fuse;
    fuse.mmax = 1;
    for (int q = 0; q < nM; ++q) fuse.mmax = M_list[q] > fuse.mmax ? M_list[q] : fuse.mmax;
    fuse.validate = orderings != NULL;
    fuse.bfl = (const int64_t *)(base + lay.bfl);
    fuse.C = C;
    fuse.bounds = bounds;
    // Where candidates share their partition DP (L > 128, few distinct link times) the schedule
    // is shared too: only the representatives are evaluated, the arg-min runs over them (a
    // representative is the lowest candidate of its group, so ties still go to the lowest
    // index), and T and C reach the other candidates only if the caller wants the arrays.
    const bool listed = lay.sh_table != 0 && pp_makespan_takes_list(S);
    const bool can_fuse = !listed && pp_makespan_can_fuse(L, D, S);
    rc = pp_launch_dp(L, D, S, N, PF, PB, XF, XB, orderings ? NULL : ord, orderings, 0,
                      can_fuse ? fuse.mmax : 0, listed, C, bounds, workspace, lay, status, st);
    if (rc) return rc;
    rc = pp_launch_makespan(L, D, S, N, nM, M_list, PF, PB, XF, XB, ord, bounds, T_all,
                            (int64_t *)(base + lay.T), status, C, base + lay.part, out,
                            (const pp_ws_header *)(base + lay.hdr), can_fuse ? &fuse : NULL,
                            listed ? (const int32_t *)(base + lay.sh_reps) : NULL, st);
    if (rc || !listed || (!T_all && !C_all)) return rc;
    return pp_launch_share_scatter(N, C_all ? 1 : 0, 0, T_all ? nM : 0, 1, C_all, NULL, T_all, workspace,
                                   lay, st);
}

extern "C" int pp_best_plan(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                            const int64_t *PB, const int64_t *XF, const int64_t *XB,
                            const int32_t *orderings, pp_result *out, int64_t *T_all,
                            int64_t *C_all, void *workspace, size_t workspace_bytes,
                            int32_t *status, void *stream) {
    if (M < 1) return PP_ERR_INVALID_ARG;
    return pp_best_plan_multi(L, D, S, N, 1, &M, PF, PB, XF, XB, orderings, out, T_all, C_all,
                              workspace, workspace_bytes, status, stream);
}

// ---------------------------------------------------------------- pp_best_plan_static
//
// pp_best_plan with the workspace in a device array that is part of the library's code
// object instead of caller memory, for callers that cannot allocate.  The array's name is
// only a host-side handle: its device address is looked up once per device (with that device
// current) and from then on only that address is used.
static __device__ __align__(256) unsigned char scratch[PP_STATIC_WORKSPACE_BYTES];

#define PP_STATIC_MAX_GPUS 64
static std::atomic<void *> scratch_at[PP_STATIC_MAX_GPUS];

static void *static_workspace() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= PP_STATIC_MAX_GPUS) return NULL;
    void *p = scratch_at[dev].load(std::memory_order_acquire);
    if (!p) {
        // every thread that gets here asks for the same address; the last store wins
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return NULL;
        scratch_at[dev].store(p, std::memory_order_release);
    }
    return p;
}

extern "C" int pp_best_plan_static(int L, int D, int S, int64_t N, int M, const int64_t *PF,
                                   const int64_t *PB, const int64_t *XF, const int64_t *XB,
                                   const int32_t *orderings, pp_result *out, int64_t *T_all,
                                   int64_t *C_all, int32_t *status, void *stream) {
    if (M < 1) return PP_ERR_INVALID_ARG;
    int rc = pp_check_sizes(L, D, S, N, orderings);
    if (rc) return rc;
    if (pp_layout(L, D, S, N).total > (size_t)PP_STATIC_WORKSPACE_BYTES) return PP_ERR_WORKSPACE;
    void *ws = static_workspace();
    if (!ws) return PP_ERR_HIP;
    return pp_best_plan_multi(L, D, S, N, 1, &M, PF, PB, XF, XB, orderings, out, T_all, C_all, ws,
                              (size_t)PP_STATIC_WORKSPACE_BYTES, status, stream);
}

extern "C" const char *pp_strerror(int code) {
    switch (code) {
        case PP_OK: return "ok";
        case PP_ERR_INVALID_ARG: return "invalid argument (NULL required pointer or size out of range)";
        case PP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case PP_ERR_HIP: return "kernel launch failed";
        default: return "unknown error code";
    }
}
