/*
 * libdpc - two-stage dynamic program for latency-aware depth compression,
 * batched, on one AMD MI355X (gfx950).  C ABI.
 *
 * The problem (paper Section 4.1-4.2, Eq. 4): a chain of L convolution layers
 * with an activation after each; choose the activations to keep, A, and the
 * merge boundaries, S, with A inside S inside {1..L-1}, maximising the summed
 * block importances I[a_{j-1}, a_j] over the chain 0 -> A -> L subject to the
 * summed block latencies T[s_{i-1}, s_i] over the chain 0 -> S -> L staying
 * within a budget T0.  The solution (Section 4.3) is two dynamic programs and
 * a walk back through their arg-min / arg-max choices; the three entry points
 * below are those three steps, each batched over B independent instances.
 *
 * Conventions common to all entry points
 *   - Every array pointer is a DEVICE pointer owned by the caller; the library
 *     allocates nothing and keeps no pointer after the call returns.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Work is queued on
 *     it and the call returns without waiting; the usual stream ordering makes
 *     the outputs of one call valid inputs of the next on the same stream.
 *   - Shapes: B >= 1 instances, 1 <= L <= DPC_MAX_L layers, P >= 1 integer
 *     latency budgets t = 0 .. P-1.  Tables indexed by two layer indices are
 *     row-major [B][L+1][L+1]; only entries [i][j] with 0 <= i < j <= L of the
 *     inputs are read.  Tables indexed by (layer, budget) are row-major
 *     [B][L+1][P].
 *   - Budgets are inclusive: column t covers total latency <= t.  The paper
 *     writes the constraint strictly (Eq. 4: latency < T0); its column T0 is
 *     column T0-1 here.
 *   - Return value: DPC_OK, or a negative DPC_ERR_* in which case nothing was
 *     queued and no output was touched.  dpc_status_string() names a code.
 *   - Calls on different streams may run concurrently as long as their output
 *     and workspace buffers are distinct.
 */
#ifndef DPC_H
#define DPC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DPC_MAX_L 255          /* layer indices and arg-max pointers fit one byte  */
#define DPC_INF   0x3FFFFFFF   /* latency of a block that cannot be merged; sums of
                                  latencies saturate at this value                 */
#define DPC_NOARG 0xFF         /* K entry of a cell that no (A, S) reaches          */

enum {
    DPC_OK          =  0,
    DPC_ERR_NULL    = -1,      /* a required pointer is NULL                        */
    DPC_ERR_SHAPE   = -2,      /* B, L, P or Q outside the supported range          */
    DPC_ERR_WORKSPACE = -3,    /* workspace smaller than dpc_stage2_workspace_bytes */
    DPC_ERR_HIP     = -4,      /* a HIP runtime call failed (launch, query)         */
    DPC_ERR_TIMEOUT = -5       /* reported by dpc_stage2_check: a bounded in-kernel
                                  wait ran out; M and K are incomplete              */
};

/* per-query status written by dpc_backtrack */
enum {
    DPC_Q_OK         = 0,
    DPC_Q_INFEASIBLE = 1,      /* no (A, S) has latency <= T0                       */
    DPC_Q_BAD_QUERY  = 2       /* q_inst outside [0,B) or q_T0 outside [0,P)        */
};

/*
 * Stage 1 - optimal merged latency of every contiguous block (Algorithm 1,
 * definitions Eq. 5a/5b):
 *     Topt[k][l] = min over S inside {k+1..l-1} of the summed T along k -> S -> l
 * computed by the algorithm's recurrence over the LAST merged block,
 *     m = lowest arg-min over k <= m' < l of  sat(Topt[k][m'] + T[m'][l]),
 * with sat(x) = min(x, DPC_INF) and Topt[k][k] = 0.
 *
 *   T      in   int32 [B][L+1][L+1]   block latency, >= 0, DPC_INF = not mergeable
 *   Topt   out  int32 [B][L+1][L+1]   entries with k >= l are written as 0
 *   split  out  uint8 [B][L+1][L+1]   the arg-min m: m == k means layers k+1..l
 *                                     stay one merged block (S_opt[k,l] empty),
 *                                     otherwise S_opt[k,l] = S_opt[k,m] + {m};
 *                                     m = k when Topt[k][l] == DPC_INF; entries
 *                                     with k >= l are written as 0
 */
int dpc_stage1_minplus(int32_t B, int32_t L, const int32_t *T, int32_t *Topt,
                       uint8_t *split, void *stream);

/*
 * Stage 2 - latency-budgeted chain DP for every budget at once (Algorithm 2,
 * recurrence Eq. 7; M is the table D of the footnote in Section 4.4):
 *     M[0][t] = +0
 *     M[j][t] = max over 0 <= i < j with Topt[i][j] <= t of
 *                   fl32( M[i][t - Topt[i][j]] + I[i][j] )
 *     K[j][t] = the lowest i attaining it
 * One IEEE binary32 add (round to nearest even, denormals kept) per
 * candidate, exact comparisons.  A cell no (A, S) reaches holds -inf and
 * K = DPC_NOARG; this carries the feasibility side condition of Eq. 7.
 *
 *   Topt   in   int32 [B][L+1][L+1]   from stage 1 (any non-negative table works)
 *   I      in   float [B][L+1][L+1]   block importance; finite or -inf (excluded
 *                                     block); NaN and +inf are not supported
 *   M      out  float [B][L+1][P]
 *   K      out  uint8 [B][L+1][P]     may be NULL: back-pointers are then not
 *                                     stored (dpc_backtrack can recompute them)
 *   workspace   device scratch of at least dpc_stage2_workspace_bytes(B, L, P)
 *               bytes, 256-byte aligned, private to this call until the work
 *               queued by it has finished; contents on entry are irrelevant
 *               (the call's own kernels clear what they need, so it can be
 *               recorded into a HIP graph)
 */
size_t dpc_stage2_workspace_bytes(int32_t B, int32_t L, int32_t P);

int dpc_stage2_knapsack(int32_t B, int32_t L, int32_t P, const int32_t *Topt,
                        const float *I, float *M, uint8_t *K, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * dpc_stage2_knapsack for callers that cannot allocate device memory or hand
 * over a workspace: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  (This entry point exists for those
 * callers; it computes nothing the one above does not.)  The workspace is a
 * fixed array of DPC_STATIC_WORKSPACE_BYTES of device memory inside the
 * library, one per GPU, held until the process ends.  The call allocates and
 * frees nothing; its first use on a GPU looks the array's address up once.
 *   - Arguments, outputs and results are those of dpc_stage2_knapsack, bit
 *     for bit, without `workspace` and `workspace_bytes`.
 *   - Shapes whose dpc_stage2_workspace_bytes(B, L, P) exceeds
 *     DPC_STATIC_WORKSPACE_BYTES are refused with DPC_ERR_WORKSPACE and
 *     nothing is queued (the five named workloads of this repository fit:
 *     the largest, B=1024, L=53, P=1000, needs 46.5 MiB).
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on
 *     a GPU (different streams, no ordering between them) race on it and must
 *     not be made; calls on one stream, or ordered by events, are fine.  What
 *     a call leaves in the array is cleared by the next call's own kernels.
 *   - A bounded wait that ran out (see dpc_stage2_check) is not reported by
 *     this variant.
 */
#define DPC_STATIC_WORKSPACE_BYTES (48u << 20)

int dpc_stage2_knapsack_static(int32_t B, int32_t L, int32_t P, const int32_t *Topt,
                               const float *I, float *M, uint8_t *K, void *stream);

/*
 * Waits for `stream` and reports whether the last dpc_stage2_knapsack that
 * used `workspace` ran to completion: DPC_OK, DPC_ERR_TIMEOUT if a bounded
 * wait inside the kernel expired (a defect or a lost device, never an input
 * property), or DPC_ERR_HIP.  Optional; the only entry point that blocks.
 */
int dpc_stage2_check(const void *workspace, void *stream);

/*
 * Set recovery - A[L,T0] and S[L,T0] (the set updates of Algorithm 2,
 * Eq. 7a/7b, and of Algorithm 1) for Q queries (instance, budget), by walking
 * the arg-max pointers K from (L, T0) down to layer 0 and, inside every block
 * (i, j) of that chain, the arg-min pointers split from j down to i.
 *
 *   Topt, split  in  as produced by stage 1
 *   I, M         in  as given to / produced by stage 2
 *   K            in  from stage 2, or NULL: the arg-max of each visited cell is
 *                    then found again as the lowest i whose candidate reproduces
 *                    the stored M bit for bit
 *   Q            number of queries, >= 0 (0: nothing is queued)
 *   q_inst,q_T0  in  int32 [Q]  instance index and inclusive budget
 *   A            out int32 [Q][L]  kept activations, ascending, A_len[q] entries
 *   S            out int32 [Q][L]  merge boundaries, ascending, S_len[q] entries,
 *                                   A is a subset of S; entries past the lengths
 *                                   are not written
 *   obj          out float [Q]     M[L][T0], the optimal objective
 *   lat          out int32 [Q]     summed latency of the chain 0 -> S -> L, <= T0
 *   status       out int32 [Q]     DPC_Q_*; for a status other than DPC_Q_OK:
 *                                   A_len = S_len = -1, obj = -inf, lat = -1
 */
int dpc_backtrack(int32_t B, int32_t L, int32_t P, const int32_t *Topt,
                  const uint8_t *split, const float *I, const float *M,
                  const uint8_t *K, int32_t Q, const int32_t *q_inst,
                  const int32_t *q_T0, int32_t *A, int32_t *A_len, int32_t *S,
                  int32_t *S_len, float *obj, int32_t *lat, int32_t *status,
                  void *stream);

/*
 * ---- Extended solver (Appendix B of the paper, "Extension on the Importance") ----
 *
 * The importance of a block now depends on whether the activations at its two
 * end points are kept: I4[k][l][a][b], a = flag at k, b = flag at l (1 = a
 * non-identity activation).  The objective is the sum of I4 along a chain
 * 0 -> B -> L of block boundaries, with flag 1 exactly at the members of A
 * (A inside B), under the same latency budget on 0 -> S -> L (A inside S).
 * Combinations a caller wants to exclude carry -inf in I4 (first lines of
 * Algorithm 3).  The flags at the two ends of the network are free.
 * Tables with flags are row-major [B][L+1][L+1][2][2].  1 <= L <= DPC_EXT_MAX_L.
 *
 * dpc_ext_importance_maxplus - Algorithm 3:
 *     Iopt[k][l][a][b] = max over chains k -> (interior points with flag 0) -> l
 *                        of the binary32 left-to-right sum of I4 along the chain,
 *     bsplit[k][l][a][b] = its last interior point m (B_opt[k,l,a,b] =
 *                        B_opt[k,m,a,0] + {m}), or k for the single block; the
 *                        single block, then the lowest m, wins ties.
 *   I4      in   float [B][L+1][L+1][2][2]   finite or -inf; only k < l is read
 *   Iopt    out  float, bsplit out uint8, same shape; entries with k >= l are 0
 */
#define DPC_EXT_MAX_L 126      /* the 2L+3 states (layer, flag) index one byte   */

int dpc_ext_importance_maxplus(int32_t B, int32_t L, const float *I4, float *Iopt,
                               uint8_t *bsplit, void *stream);

/*
 * dpc_ext_knapsack - Algorithm 4 for every budget at once:
 *     D[0][t][a] = +0,
 *     D[l][t][a] = max over k' < l, alpha' in {0,1}, Topt[k'][l] <= t of
 *                  fl32( D[k'][t - Topt[k'][l]][alpha'] + Iopt[k'][l][alpha'][a] ),
 *     the lowest (k', alpha') attaining it is kept as 2k' + alpha'.
 * It runs as the stage-2 recurrence on the chain of states v = 2l + a:
 *   D    out  float [B][2L+3][P]   row 2l+a is D[l][.][a]; the last row, 2L+2,
 *                                  is max over a of D[L][.][a] (the solution)
 *   Kx   out  uint8 [B][2L+3][P]   row 2l+a: 2k'+alpha' of the arg-max; last
 *                                  row: 2L + a_last; DPC_NOARG where nothing
 *                                  reaches; must not be NULL for dpc_ext_backtrack
 *   Topt in   from dpc_stage1_minplus;  Iopt in  from dpc_ext_importance_maxplus
 *   workspace   at least dpc_ext_workspace_bytes(B, L, P) bytes, 256-byte
 *               aligned, private to the call while its work is queued
 * dpc_ext_check is dpc_stage2_check for such a workspace.
 */
size_t dpc_ext_workspace_bytes(int32_t B, int32_t L, int32_t P);

int dpc_ext_knapsack(int32_t B, int32_t L, int32_t P, const int32_t *Topt, const float *Iopt,
                     float *D, uint8_t *Kx, void *workspace, size_t workspace_bytes,
                     void *stream);

int dpc_ext_check(int32_t B, int32_t L, int32_t P, const void *workspace, void *stream);

/*
 * dpc_ext_backtrack - the sets of Algorithm 4 for Q queries (instance, budget):
 * A (activations kept), S (merge boundaries, A inside S) and B (block
 * boundaries of the objective, A inside B), each ascending in int32 [Q][L]
 * with its length; obj = D[L][T0][a_last], a_last = the better final flag
 * (lowest on ties), lat = summed latency of 0 -> S -> L.  status and the
 * values for a status other than DPC_Q_OK are as in dpc_backtrack.
 */
int dpc_ext_backtrack(int32_t B, int32_t L, int32_t P, const int32_t *Topt,
                      const uint8_t *split, const uint8_t *bsplit, const float *D,
                      const uint8_t *Kx, int32_t Q, const int32_t *q_inst,
                      const int32_t *q_T0, int32_t *A, int32_t *A_len, int32_t *S,
                      int32_t *S_len, int32_t *Bs, int32_t *B_len, float *obj,
                      int32_t *lat, int32_t *a_last, int32_t *status, void *stream);

/* Name of a DPC_ERR_* code (static string, never NULL). */
const char *dpc_status_string(int code);

/*
 * ---- Small instances: stage 1 and stage 2 in one launch ----
 *
 * dpc_stage12_fused computes exactly what dpc_stage1_minplus followed by
 * dpc_stage2_knapsack computes (Algorithms 1 and 2; same outputs, bit for
 * bit), in a single kernel with one workgroup per instance that keeps the
 * tables of an instance in LDS.  It is the low-latency path for one network or
 * a few of them; it needs no workspace and cannot time out (no workgroup waits
 * for another).  Follow it with dpc_backtrack.
 * Supported shapes: 1 <= L <= 63, 1 <= P <= 2048 and a device whose LDS holds
 * the candidate table and at least one row of M (true for every such shape on
 * MI355X); dpc_stage12_fused_supported returns 1 for them on the current
 * device, else 0, and dpc_stage12_fused returns DPC_ERR_SHAPE for the others.
 *   T, I            in   as for dpc_stage1_minplus / dpc_stage2_knapsack
 *   Topt, split     out  as written by dpc_stage1_minplus
 *   M, K            out  as written by dpc_stage2_knapsack; K may be NULL
 */
int dpc_stage12_fused_supported(int32_t L, int32_t P);

int dpc_stage12_fused(int32_t B, int32_t L, int32_t P, const int32_t *T, const float *I,
                      int32_t *Topt, uint8_t *split, float *M, uint8_t *K, void *stream);

/*
 * dpc_solve_fused - the whole path (Algorithms 1 and 2 and the set recovery of
 * dpc_backtrack) in ONE launch: dpc_stage12_fused, after which the workgroup of
 * an instance goes on to answer the queries that name that instance, one wave
 * per query at a time.  Outputs are those of dpc_stage12_fused followed by
 * dpc_backtrack, bit for bit (a query that names no instance gets
 * DPC_Q_BAD_QUERY as there).  It saves a launch when there are few queries
 * per instance (one network, one budget: the paper's use); with many queries
 * per instance the separate dpc_backtrack, which spreads them over the whole
 * chip, is faster.  Shapes as for dpc_stage12_fused; Q >= 0 (0: no queries).
 */
int dpc_solve_fused(int32_t B, int32_t L, int32_t P, const int32_t *T, const float *I,
                    int32_t *Topt, uint8_t *split, float *M, uint8_t *K, int32_t Q,
                    const int32_t *q_inst, const int32_t *q_T0, int32_t *A, int32_t *A_len,
                    int32_t *S, int32_t *S_len, float *obj, int32_t *lat, int32_t *status,
                    void *stream);

/*
 * ---- Steps around the solver in a sweep over hyper-parameters ----
 *
 * dpc_importance_shift - the normalisation of the paper's appendix "Evaluating
 * and Normalizing the Importance": every block's importance is lowered by
 * alpha times the mean importance of the blocks of size one,
 *     I_out[b][a][.] = fl32( I_raw[b][.] - alpha[a] * mean_b ),
 *     mean_b = mean of the finite entries I_raw[b][i][i+1][f], 0 <= i < L
 *              (0 when there is none),
 * for every raw table b and every alpha a: B * n_alpha tables come out, table
 * b * n_alpha + a belonging to (b, a), ready to be solved as that many
 * instances.  The mean is accumulated in binary64 in ascending (i, f), the
 * product and the difference are binary64 operations, the result is rounded to
 * binary32 once.  -inf entries (excluded blocks) stay -inf.
 *   F         1: tables [L+1][L+1];  4: tables with flags [L+1][L+1][2][2]
 *   I_raw     in   float [B][L+1][L+1][F]
 *   alpha     in   float [n_alpha]            device memory, 0 <= n_alpha <= 65535
 *   I_out     out  float [B][n_alpha][L+1][L+1][F]   every entry is written
 *   mean_out  out  double [B], or NULL
 */
int dpc_importance_shift(int32_t B, int32_t L, int32_t F, int32_t n_alpha, const float *I_raw,
                         const float *alpha, float *I_out, double *mean_out, void *stream);

/*
 * Shared stage-1 tables.  In a sweep over the normalisation constant the B
 * instances are `share` consecutive copies of each network (instance x is
 * network x / share, as dpc_importance_shift lays them out): their latency
 * tables are the same, so stage 1 has to run once per network only.
 * dpc_stage2_knapsack_shared and dpc_backtrack_shared are dpc_stage2_knapsack
 * and dpc_backtrack with
 *   Topt, split   in  [ceil(B / share)][L+1][L+1]: table x / share serves instance x
 * and every other argument (I, M, K, the queries and the outputs, all per
 * instance) unchanged.  share >= 1; share = 1 is the plain call.
 */
int dpc_stage2_knapsack_shared(int32_t B, int32_t L, int32_t P, int32_t share,
                               const int32_t *Topt, const float *I, float *M, uint8_t *K,
                               void *workspace, size_t workspace_bytes, void *stream);

int dpc_backtrack_shared(int32_t B, int32_t L, int32_t P, int32_t share, const int32_t *Topt,
                         const uint8_t *split, const float *I, const float *M,
                         const uint8_t *K, int32_t Q, const int32_t *q_inst,
                         const int32_t *q_T0, int32_t *A, int32_t *A_len, int32_t *S,
                         int32_t *S_len, float *obj, int32_t *lat, int32_t *status,
                         void *stream);

/*
 * dpc_front - the latency/objective trade-off curve of an instance, read off
 * the last row of the table of Algorithm 2: the budgets t at which the optimum
 * of Eq. 4 improves, M[L][t] > M[L][t-1] (column -1 counting as -inf).  At
 * such a t the optimal (A, S) has latency exactly t; between two of them the
 * solution does not change, so these are the only budgets a sweep over T0
 * needs to recover sets for.
 *   M          in   float [B][L+1][P]   from dpc_stage2_knapsack; only row L is
 *                                       read.  For the table D of
 *                                       dpc_ext_knapsack pass 2L+2 in place of L.
 *   cap             room per instance in front_t / front_obj, >= 0
 *   front_t    out  int32 [B][cap]      budgets, ascending
 *   front_obj  out  float [B][cap]      M[L][t] at those budgets
 *   front_len  out  int32 [B]           number of points of the curve; when it
 *                                       exceeds cap only the first cap are
 *                                       written.  Entries past the points
 *                                       written are left untouched.
 */
int dpc_front(int32_t B, int32_t L, int32_t P, const float *M, int32_t cap, int32_t *front_t,
              float *front_obj, int32_t *front_len, void *stream);

/*
 * dpc_front_queries - the points of the curves of a batch as one list of
 * queries (instance, budget), instance by instance, budgets ascending: the
 * budgets a sweep over T0 has to recover sets for (pass the list to
 * dpc_backtrack; a budget between two points has the solution of the point
 * below it).
 *   front_t, front_len   in   as written by dpc_front with the same cap; an
 *                             instance contributes min(front_len, cap) points
 *   qcap                      room in q_inst / q_T0, >= 0
 *   q_inst, q_T0         out  int32 [qcap]
 *   q_count              out  int32 [1]   number of queries in all; when it
 *                             exceeds qcap only the first qcap are written
 */
int dpc_front_queries(int32_t B, int32_t cap, const int32_t *front_t, const int32_t *front_len,
                      int32_t qcap, int32_t *q_inst, int32_t *q_T0, int32_t *q_count,
                      void *stream);

/*
 * dpc_chain_latency - latency of the network merged at a given ordered set X:
 * the sum of T over consecutive members of 0 -> X -> L, saturating at DPC_INF
 * (the constraint side of Eq. 4 with X in place of S).  With X = S of
 * dpc_backtrack it reproduces lat; with X = A it is the latency of merging at
 * the kept activations only, the comparison of the paper's ablation on the
 * ordered set to be merged.
 *   T       in   int32 [B][L+1][L+1]
 *   q_inst  in   int32 [Q]      instance of each query
 *   X       in   int32 [Q][L]   members ascending in [1, L-1], X_len[q] of them
 *   X_len   in   int32 [Q]
 *   lat     out  int32 [Q]      -1 for X_len < 0 (the "no solution" marker of
 *                               dpc_backtrack), for an instance outside [0, B)
 *                               and for a set that is not ascending in [1, L-1]
 */
int dpc_chain_latency(int32_t B, int32_t L, const int32_t *T, int32_t Q, const int32_t *q_inst,
                      const int32_t *X, const int32_t *X_len, int32_t *lat, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DPC_H */
