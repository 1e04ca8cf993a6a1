/*
 * dssync.h -- C ABI of the MI355X (gfx950) DS-Sync hot path.
 *
 * One DS-Sync synchronisation step over W simulated worker replicas that are
 * stacked, one row per worker, in one GPU's HBM:
 *
 *   1. ds_partition        divide the workers into non-overlapping groups for
 *                          iteration t                       (host, integer)
 *   2. ds_group_sync       every worker applies its local SGD update, then the
 *      ds_group_sync_ragged  updated parameters are averaged inside each group
 *                          and the mean is written back to every member (GPU)
 *   3. ds_consensus        distance of every replica from the mean replica (GPU)
 *
 * Conventions shared by every entry point
 *   - Return value: DS_OK (0) or a negative ds_status.  Nothing throws or aborts.
 *   - All argument checks run on the host BEFORE the first HIP call, so every
 *     error other than DS_ERR_HIP is reported without touching a GPU, and a
 *     call that returns an error has enqueued nothing.
 *   - "dev" pointers are device memory on the current HIP device, "host"
 *     pointers ordinary host memory.  Every buffer is owned by the caller.
 *     Host arrays are consumed before the call returns.  Device buffers must
 *     stay valid until `stream` has executed the enqueued work.
 *   - GPU work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No entry point synchronises, allocates or frees
 *     device memory, except ds_ragged_plan (a one-off set-up call, see there).
 *   - The library keeps no state between calls.
 *   - Row-major stacks: element (worker i, column p) of a stack with leading
 *     dimension ld is at base + i*ld + p, ld >= P.  Replica stacks are fp32.
 */
#ifndef DSSYNC_H
#define DSSYNC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DS_OK            =  0,
    DS_ERR_NULL      = -1,  /* a required pointer is NULL                                  */
    DS_ERR_BAD_W     = -2,  /* W outside 1..DS_MAX_W                                       */
    DS_ERR_BAD_SIZES = -3,  /* group sizes: n_groups < 1, a size < 1, or sum != W          */
    DS_ERR_BAD_PART  = -4,  /* perm is not a permutation of 0..W-1, or off is not 0..W
                               strictly increasing                                         */
    DS_ERR_BAD_SHAPE = -5,  /* P < 0, ld < P, bad segment table, size overflow             */
    DS_ERR_ALIGN     = -6,  /* base pointer, leading dimension or segment offset breaks
                               the alignment rule stated at the entry point                */
    DS_ERR_DTYPE     = -7,  /* g_dtype is neither DS_F32 nor DS_BF16                       */
    DS_ERR_WORKSPACE = -8,  /* workspace / plan buffer NULL, misaligned or too small       */
    DS_ERR_HIP       = -9,  /* a HIP call or kernel launch failed                          */
    DS_ERR_TOPOLOGY  = -10  /* rack table: index outside 0..n_racks-1, an unused rack index,
                               or a rack whose workers all have NIC contention             */
} ds_status;

/* gradient element type */
enum { DS_F32 = 0, DS_BF16 = 1 };

/* Largest number of workers.  The division of the workers travels inside the
   kernel-argument block, so no host-to-device copy sits on the path. */
#define DS_MAX_W 64

/* Human-readable name of a status code (static storage, never NULL). */
const char* ds_status_string(int status);

/*
 * ds_partition -- the group of every worker in iteration t.
 *
 * Paper: Listing 1 ("pick the proper group to synchronize for worker i in the
 * iteration t") and Sec. IV-B2 (each iteration's groups are disjoint and cover
 * all workers; groups may differ in size, Sec. III-A).  The paper's list is
 * derived from the network topology; this routine draws iteration t's entry
 * with a counter-based shuffle instead, so any (seed, t) can be evaluated in
 * any order and nothing is carried between iterations:
 *     gamma = 0x9E3779B97F4A7C15, mix = splitmix64 finaliser
 *     s = mix(mix(seed) + (t+1)*gamma);  each draw: s += gamma, r = mix(s)
 *     perm = identity; for i = W-1 .. 1: j = floor(r*(i+1) / 2^64), swap perm[i], perm[j]
 * Group k is perm_out[off_out[k] .. off_out[k+1]-1] with off_out the prefix
 * sums of sizes.
 *
 *   seed, t     shuffle key and iteration number
 *   W           number of workers, 1..DS_MAX_W
 *   sizes       host [n_groups], each >= 1, summing to W
 *   perm_out    host [W], written
 *   off_out     host [n_groups+1], written
 * Host only: integer arithmetic, no GPU call.
 * Errors: DS_ERR_NULL, DS_ERR_BAD_W, DS_ERR_BAD_SIZES.
 */
int ds_partition(uint64_t seed, uint64_t t, int32_t W, const int32_t* sizes, int32_t n_groups,
                 int32_t* perm_out, int32_t* off_out);

/*
 * ds_pattern -- the paper's own divide-and-shuffle pattern for iteration t,
 * from the rack of every worker (a second source of divisions next to
 * ds_partition; the output feeds ds_group_sync unchanged).
 *
 * Paper: Sec. III-B.  (1) Static topology: the workers of a rack form an
 * intra-rack group except one representative per rack; the representatives
 * form the inter-rack group, so every rack has one connection on its
 * inter-rack link; the workers of a rack take turns as representative.
 * (2) Inter-rack link contention: the representative of a delayed rack is
 * paired with one regular representative (group of two), the other regular
 * representatives form the large inter-rack group, and the regular partner
 * changes every iteration.  (3) End-host NIC contention: a delayed worker is
 * never a representative; it is paired with one regular worker of its rack
 * (group of two, partner changing every iteration) while the rest of the rack
 * forms the large intra-rack group.
 * The prose leaves the rotations open; the ones used (t is the only state):
 *   representative of rack r   = free_r[t mod |free_r|], free_r = workers of r
 *                                without NIC contention, ascending index;
 *   partner of k-th delayed rack = regular[(t+k) mod |regular|] (ascending rack
 *                                index); delayed racks beyond the number of
 *                                regular ones are paired among themselves; if
 *                                no rack or every rack is delayed, all
 *                                representatives form one group;
 *   partner of k-th delayed worker of a rack = fast[(t+k) mod |fast|], fast =
 *                                regular non-representatives of the rack; the
 *                                rack is split only if |fast| > number of
 *                                delayed workers (someone is left for the hub).
 * With a single rack nobody is set apart (one group: plain BSP).
 * Group order: inter-rack pairs, large inter-rack group, then per rack its
 * pairs and its large group.
 *
 *   W            workers, 1..DS_MAX_W
 *   rack_of      host [W], rack index of every worker, 0..n_racks-1, every index used
 *   slow_rack    host [n_racks], non-zero = contention on that rack's inter-rack link
 *   slow_worker  host [W], non-zero = contention on that worker's NIC
 *   t            iteration
 *   perm_out     host [W], off_out host [W+1] (at most W groups), n_groups_out: written
 * ds_pattern_period writes a period B of the pattern: the division of
 * iteration t+B equals that of t (Sec. IV-B2: W_k = W_{k+B}).
 * Host only.  Errors: DS_ERR_NULL, DS_ERR_BAD_W, DS_ERR_TOPOLOGY.
 */
int ds_pattern(int32_t W, const int32_t* rack_of, const uint8_t* slow_rack, int32_t n_racks,
               const uint8_t* slow_worker, uint64_t t, int32_t* perm_out, int32_t* off_out,
               int32_t* n_groups_out);

int ds_pattern_period(int32_t W, const int32_t* rack_of, const uint8_t* slow_rack, int32_t n_racks,
                      const uint8_t* slow_worker, uint64_t* period_out);

/*
 * ds_group_sync -- local SGD update fused with the in-group parameter average.
 *
 * Paper: Listing 1, optimizer.step() followed by Average(model, group);
 * Sec. III-A step 4 (parameters are averaged within the group after the local
 * update); Sec. IV-B2, X_{k+1} = W_k X_k with w_ij = 1/|group|.
 * For every group g and column p < P:
 *     m = (1/|g|) * sum_{i in g} ( X[i,p] - lr * G[i,p] );   X[i,p] = m for all i in g
 * One value is computed per (group, column) and stored |g| times, so the rows
 * of a group are bit-identical afterwards.  fp32 arithmetic; bf16 gradients
 * are widened exactly.  Each replica element is read once and written once.
 *
 *   X        dev fp32 [W, ldx], in/out, updated in place
 *   G        dev [W, ldg], fp32 (DS_F32) or bf16 (DS_BF16), read only,
 *            must not overlap X
 *   P        columns to process, >= 0 (0 enqueues nothing)
 *   ldx,ldg  leading dimensions in elements, >= P, multiples of 4
 *   perm,off host; any valid division of the workers (as ds_partition writes it,
 *            or any other: the call does not care how the groups were chosen)
 *   lr       learning rate
 * Alignment: X and G 16-byte aligned.  Fastest with 1-KiB-aligned bases and
 * ldx = ldg = ds_padded_ld(P) (every row on a 1-KiB boundary).
 * Errors: DS_ERR_NULL, DS_ERR_BAD_W, DS_ERR_BAD_SIZES, DS_ERR_BAD_PART,
 *         DS_ERR_BAD_SHAPE, DS_ERR_ALIGN, DS_ERR_DTYPE, DS_ERR_HIP.
 */
int ds_group_sync(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx, int64_t ldg,
                  int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups, float lr,
                  void* stream);

/*
 * Ragged variant: the same step over S column segments of the stacks in ONE
 * launch.  Paper: Sec. V-A1 (parameters are synchronised layer by layer) and
 * Sec. IV-A (the model is synchronised L times per iteration); a segment is
 * one layer's slice of every replica.  Columns outside the segments are left
 * untouched.
 *
 * A segment is columns offset .. offset+length-1 of every row.  Rules: length
 * >= 0 (empty segments are allowed), offset >= 0 and a multiple of 8 elements
 * (fastest: a multiple of 256, so that segments start on 1-KiB boundaries),
 * offset+length <= min(ldx, ldg), segments pairwise disjoint.
 *
 * The segment list is turned once into a device-side tile table ("plan"):
 *   ds_ragged_plan_bytes   bytes the plan needs (0 if every segment is empty)
 *   ds_ragged_plan         builds the table on the host, copies it to `plan`
 *                          on `stream` and WAITS for the copy (set-up call,
 *                          once per layer list)
 *   ds_group_sync_ragged   kernel launch only; `segs`/`S` must be the list the
 *                          plan was built from (only its tile count is re-derived)
 * plan: dev, 16-byte aligned, at least ds_ragged_plan_bytes bytes.
 * Other arguments, alignment and errors as ds_group_sync; a bad segment table
 * is DS_ERR_BAD_SHAPE (or DS_ERR_ALIGN for an offset), a bad plan buffer
 * DS_ERR_WORKSPACE.
 */
typedef struct {
    int64_t offset;  /* first column, in elements */
    int64_t length;  /* number of columns         */
} ds_segment;

size_t ds_ragged_plan_bytes(const ds_segment* segs, int32_t S);

int ds_ragged_plan(const ds_segment* segs, int32_t S, int64_t ldx, int64_t ldg, void* plan,
                   size_t plan_bytes, void* stream);

int ds_group_sync_ragged(void* X, const void* G, int32_t g_dtype, const ds_segment* segs, int32_t S,
                         int64_t ldx, int64_t ldg, int32_t W, const int32_t* perm,
                         const int32_t* off, int32_t n_groups, float lr, const void* plan,
                         size_t plan_bytes, void* stream);

/*
 * ds_group_sync_opt / ds_group_sync_ragged_opt -- the same step with the fuller
 * local optimizer and the SWA ensemble.
 *
 * Paper: Listing 1 (optimizer.step(); Average(model, group); SWA_model =
 * factor*SWA_model + (1-factor)*model) and Sec. V-A3 (hyper-parameters of the
 * original model papers, i.e. SGD with momentum and weight decay for the
 * WideResNets).  Only the model is handed to Average, so the momentum buffer
 * stays local to its worker and is never averaged.  Per worker i, column p:
 *     d  = G[i,p] + weight_decay * X[i,p]
 *     v' = momentum * V[i,p] + d;  V[i,p] = v'       (V == NULL: v' = d)
 *     y_i = X[i,p] - lr * v'
 * then m = mean of the y_i over the group, X[i,p] = m for every member, and
 *     S[i,p] = swa_factor * S[i,p] + (1 - swa_factor) * m      (S != NULL)
 * all in the one fused pass: V and S add a read and a write of 4 bytes each
 * per (worker, column).  opt == NULL, or V == S == NULL with weight_decay == 0,
 * is exactly ds_group_sync.  The final model of Listing 1 (average of all SWA
 * models) is one ds_group_sync over S with a single group of W workers, a zero
 * gradient stack and lr = 0.
 *   V, S     dev fp32 [W, ldv] / [W, lds], in/out, 16-byte aligned, leading
 *            dimension >= P (ragged: >= end of the last segment) and a
 *            multiple of 4; must not overlap X, G or each other
 * Other arguments and errors as ds_group_sync / ds_group_sync_ragged.
 */
typedef struct {
    void*   V;             /* momentum buffers, or NULL                       */
    int64_t ldv;
    float   momentum;      /* used only when V != NULL                        */
    float   weight_decay;
    void*   S;             /* SWA models, or NULL                             */
    int64_t lds;
    float   swa_factor;    /* used only when S != NULL                        */
} ds_local_opt;

int ds_group_sync_opt(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx, int64_t ldg,
                      int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups, float lr,
                      const ds_local_opt* opt, void* stream);

int ds_group_sync_ragged_opt(void* X, const void* G, int32_t g_dtype, const ds_segment* segs, int32_t S,
                             int64_t ldx, int64_t ldg, int32_t W, const int32_t* perm,
                             const int32_t* off, int32_t n_groups, float lr, const ds_local_opt* opt,
                             const void* plan, size_t plan_bytes, void* stream);

/*
 * ds_consensus -- how far every replica is from the mean replica.
 *
 * Paper: Sec. IV-B2; the left-hand side of Lemma 1 for worker i, un-squared:
 *     xbar[p] = (1/W) * sum_i X[i,p];   dev_out[i] = sqrt( sum_{p<P} (X[i,p] - xbar[p])^2 )
 * The column mean and the differences are formed in fp64, so identical
 * replicas give exactly 0.  The result is deterministic (fixed reduction
 * tree, no floating-point atomics).  X is read once.
 *
 *   X          dev fp32 [W, ld], read only; 16-byte aligned, ld >= P, ld % 4 == 0
 *   dev_out    dev fp64 [W], written
 *   workspace  dev, 16-byte aligned, >= ds_consensus_workspace_bytes(W, P) bytes,
 *              overwritten (per-block partial sums)
 * P == 0 writes zeros.
 * Errors: DS_ERR_NULL, DS_ERR_BAD_W, DS_ERR_BAD_SHAPE, DS_ERR_ALIGN,
 *         DS_ERR_WORKSPACE, DS_ERR_HIP.
 */
size_t ds_consensus_workspace_bytes(int32_t W, int64_t P);

int ds_consensus(const void* X, int64_t P, int64_t ld, int32_t W, double* dev_out, void* workspace,
                 size_t workspace_bytes, void* stream);

/*
 * ds_consensus_grouped -- the same norms for a stack whose rows are known to be
 * identical inside every group of the given division, which is the state
 * right after ds_group_sync* with that division (Listing 1: members leave
 * Average with the same model).  Only one row per group is read
 * (4*n_groups*P bytes instead of 4*W*P); with m_k that row and n_k = |g_k|:
 *     xbar[p] = (1/W) * sum_k n_k * m_k[p];   dev_out[i] = || m_{g(i)} - xbar ||_2
 * PRECONDITION, not checked: rows of a group are equal.  If they are not, the
 * result describes the stack in which every member is replaced by its group's
 * first member.  Arguments, workspace and errors as ds_consensus, plus those
 * of a division (DS_ERR_BAD_SIZES, DS_ERR_BAD_PART).
 */
int ds_consensus_grouped(const void* X, int64_t P, int64_t ld, int32_t W, const int32_t* perm,
                         const int32_t* off, int32_t n_groups, double* dev_out, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * ds_padded_ld -- the leading dimension (row pitch, in elements) the kernels
 * run fastest with for rows of P elements: P rounded up to an odd multiple of
 * 256.  Data layout only, not a step of the method (the paper stacks the
 * replicas as the rows of X_k, Sec. IV-B2, and says nothing of a pitch).
 * Every row of an fp32 stack then starts on a 1-KiB boundary, so each 1-KiB
 * wavefront access covers one aligned KiB of its row (measured 2-5 % faster
 * on MI355X than rows starting on other 256-byte boundaries, 15-20 % faster
 * than a dense pitch whose rows straddle cache lines), and the odd multiple
 * keeps the pitch away from large powers of two, where equal columns of
 * different rows fall on the same memory channels.  Any ld >= P that is a
 * multiple of 4 is accepted by every entry point; this one is a recommendation.
 * Host only.  Returns 0 if P < 0 or the result would not fit in int64_t.
 */
int64_t ds_padded_ld(int64_t P);

/*
 * ds_probe_copy -- measurement aid, not a step of the method: a plain
 * device-to-device streaming copy of `bytes` bytes (reads `bytes`, writes
 * `bytes`).  The benchmark uses it as the attainable-bandwidth yardstick and
 * to scale the profiler's HBM byte counters against a launch whose traffic is
 * known exactly.
 *   dst, src   dev, 16-byte aligned, non-overlapping; bytes a multiple of 16
 * Errors: DS_ERR_NULL, DS_ERR_ALIGN, DS_ERR_BAD_SHAPE, DS_ERR_HIP.
 */
int ds_probe_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DSSYNC_H */
