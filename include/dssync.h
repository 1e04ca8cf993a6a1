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
 *     the default stream).  No entry point synchronises, copies between host
 *     and device, or allocates or frees device memory: a GPU entry point
 *     issues kernel launches and nothing else, so each of them can be
 *     recorded into a HIP graph.
 *   - The library keeps no state between calls, apart from two attributes of
 *     each device (number of compute units, LDS per compute unit), which are
 *     read once per process and device on the first launch there, and the
 *     per-device address of the array ds_consensus_static works in.
 *   - One launch covers at most DS_MAX_COLUMNS columns; longer rows are
 *     DS_ERR_BAD_SHAPE (columns are independent, so the caller can split them).
 *   - Row-major stacks: element (worker i, column p) of a stack with leading
 *     dimension ld is at base + i*ld + p, ld >= P.  Replica stacks are fp32.
 *     (A second, tiled layout with entry points of its own is described at
 *     the end of this file.)
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
    DS_ERR_TOPOLOGY  = -10, /* rack table: index outside 0..n_racks-1, an unused rack index,
                               or a rack whose workers all have NIC contention             */
    DS_ERR_HOST_MEMORY = -11 /* a host-side allocation inside the call failed              */
} ds_status;

/* gradient element type */
enum { DS_F32 = 0, DS_BF16 = 1 };

/* Largest number of workers.  The division of the workers travels inside the
   kernel-argument block, so no host-to-device copy sits on the path. */
#define DS_MAX_W 64

/* Largest number of columns one launch covers: the grid of one-wavefront
   workgroups of 256 columns must stay below HIP's limit of 2^32 threads along
   x (about 17.18e9 columns, 68.7 GB per fp32 row). */
#define DS_MAX_COLUMNS ((((int64_t)1 << 26) - 1) * 256)

/* Human-readable name of a status code (static storage, never NULL). */
const char* ds_status_string(int status);

/*
 * ds_partition -- the group of every worker in iteration t.
 *
 * Paper: Listing 1 (the per-iteration lookup of worker i's group in the group
 * list) and Sec. IV-B2 (each iteration's groups are disjoint and cover
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
 * ds_pattern_check -- does a periodic list of divisions meet the premise of
 * the paper's consensus bound, and how fast does it contract?
 *
 * Paper: Sec. IV-B2.  Division k of the period has the mixing matrix W_k
 * (w_ij = 1/|group| for two members of one group, else 0) and one period is
 * M = W_{B-1} ... W_0.  Lemma 1 requires the period to be connected (the
 * union, over the period, of the groups taken as complete graphs is a single
 * component) and bounds the consensus error after k periods by rho^k with rho
 * the second largest eigenvalue modulus of M.  This routine reports
 *   connected_out  1 if the union graph is one component, else 0 (union-find
 *                  over the groups of the period);
 *   rho_out        the spectral radius of M - 11^T/W, i.e. that second
 *                  eigenvalue modulus (M is a product of symmetric matrices
 *                  but not symmetric itself, so its eigenvalues may be
 *                  complex; the radius is taken as lim ||A^(2^j)||^(1/2^j) by
 *                  repeated squaring in fp64, accurate to about 1e-12);
 *   sigma_out      || M - 11^T/W ||_2 >= rho, the factor by which one period
 *                  is guaranteed to shrink || X - mean ||_F for every X (the
 *                  square root of the spectral radius of A^T A, same method).
 * rho < 1, sigma < 1 and connected are equivalent (every W_k is an orthogonal
 * projector, so ||M x|| = ||x|| only for x constant on every component).
 * The list may come from ds_pattern, ds_partition or anywhere else.
 *
 *   W          workers, 1..DS_MAX_W
 *   B          divisions in the period, >= 1
 *   perms      host [B*W]:     perm of division k at perms + k*W
 *   offs       host [B*(W+1)]: off of division k at offs + k*(W+1), the first
 *              n_groups[k]+1 entries used
 *   n_groups   host [B]
 *   rho_out, sigma_out  may each be NULL (that part is then skipped)
 * Host only, fp64, O(B*W^2 + W^3) work, no allocation.
 * Errors: DS_ERR_NULL, DS_ERR_BAD_W, DS_ERR_BAD_SHAPE (B < 1), DS_ERR_BAD_SIZES,
 *         DS_ERR_BAD_PART (a list entry is not a division of the workers).
 */
int ds_pattern_check(int32_t W, int32_t B, const int32_t* perms, const int32_t* offs,
                     const int32_t* n_groups, int32_t* connected_out, double* rho_out,
                     double* sigma_out);

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
 *   ds_ragged_plan         set-up call, once per layer list: checks the list
 *                          and enqueues small kernels on `stream` that write
 *                          the table (the segments travel in the kernel
 *                          arguments, 96 per launch: no copy, no wait).
 *                          *plan_id_out receives the identity of the plan, a
 *                          hash of the segment list that is never 0 (0 if the
 *                          list has no columns); it is also stored in the
 *                          plan's first entry.
 *   ds_group_sync_ragged   kernel launch only.  `segs`/`S` must be the list
 *                          the plan was built from and `plan_id` the value
 *                          ds_ragged_plan returned for this buffer: a plan_id
 *                          that is not that of `segs` is DS_ERR_WORKSPACE,
 *                          reported on the host before anything is enqueued.
 *                          On the device every workgroup compares plan_id and
 *                          the entry count with the plan's first entry and
 *                          leaves the stacks untouched if they differ (a
 *                          buffer that holds another plan, or none), and an
 *                          entry that points outside the rows is skipped.
 * plan: dev, 16-byte aligned, at least ds_ragged_plan_bytes bytes; it must not
 * be written by anyone else while launches that use it are pending.
 * Other arguments, alignment and errors as ds_group_sync; a bad segment table
 * is DS_ERR_BAD_SHAPE (or DS_ERR_ALIGN for an offset), a bad plan buffer or
 * plan_id DS_ERR_WORKSPACE, a list whose lengths, each rounded up to a
 * multiple of 2048 columns, add up to more than DS_MAX_COLUMNS
 * DS_ERR_BAD_SHAPE; ds_ragged_plan may also return DS_ERR_HOST_MEMORY (its
 * overlap check sorts a host copy of the list).
 */
typedef struct {
    int64_t offset;  /* first column, in elements */
    int64_t length;  /* number of columns         */
} ds_segment;

size_t ds_ragged_plan_bytes(const ds_segment* segs, int32_t S);

int ds_ragged_plan(const ds_segment* segs, int32_t S, int64_t ldx, int64_t ldg, void* plan,
                   size_t plan_bytes, uint64_t* plan_id_out, void* stream);

int ds_group_sync_ragged(void* X, const void* G, int32_t g_dtype, const ds_segment* segs, int32_t S,
                         int64_t ldx, int64_t ldg, int32_t W, const int32_t* perm,
                         const int32_t* off, int32_t n_groups, float lr, const void* plan,
                         size_t plan_bytes, uint64_t plan_id, void* stream);

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
                             const void* plan, size_t plan_bytes, uint64_t plan_id, void* stream);

/*
 * ds_consensus -- how far every replica is from the mean replica.
 *
 * Paper: Sec. IV-B2; the left-hand side of Lemma 1 for worker i, un-squared:
 *     xbar[p] = (1/W) * sum_i X[i,p];   dev_out[i] = sqrt( sum_{p<P} (X[i,p] - xbar[p])^2 )
 * Arithmetic: the column mean is formed in fp64 and split into an fp32 pair
 * hi + lo; the difference (x - hi) - lo and its square are fp32, so the
 * rounding error is relative to the difference itself and identical replicas
 * give exactly 0.  A lane sums the squares of at most 256 columns per worker
 * in fp32 before the sum is widened; everything above that (across lanes,
 * wavefronts, workgroups) is fp64.  Relative error of a norm: below 8e-6 in the
 * worst case and about 5e-7 typically, whatever P.  The result is
 * deterministic (fixed reduction tree, no floating-point atomics).  X is read
 * once.
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
 * ds_consensus_static -- ds_consensus without a workspace argument, for callers
 * that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The per-workgroup partial
 * sums go to an array that is part of the library's device image (4 MiB:
 * 8192 partial rows of DS_MAX_W fp64 sums, the largest workspace ds_consensus
 * ever asks for), held by every GPU the library runs on until the process
 * ends.  The call allocates and frees nothing and calls no routine that does.
 * Same kernels and same result, bit for bit, as ds_consensus.
 *
 * Limits: the array covers every W <= DS_MAX_W and every P <= DS_MAX_COLUMNS
 * (a workgroup walks as many column tiles as it takes to stay within 8192
 * workgroups); anything larger is refused as in ds_consensus (DS_ERR_BAD_W,
 * DS_ERR_BAD_SHAPE).  The first call on a device looks up the array's address
 * there (hipGetSymbolAddress, with that device current) and keeps it; make that
 * first call outside stream capture.  The array keeps the last call's partial
 * sums; every launch overwrites all the entries it later reads, so nothing has
 * to be cleared.  All calls on one GPU share the one array: two calls whose
 * kernels may run at the same time (different streams, or graphs launched
 * side by side) race and give wrong norms; order them on one stream or with
 * events.
 * Arguments and errors as ds_consensus without the workspace;
 * DS_ERR_HIP also if the array's address cannot be obtained.
 */
int ds_consensus_static(const void* X, int64_t P, int64_t ld, int32_t W, double* dev_out, void* stream);

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
 * ds_group_sync_consensus -- ds_group_sync and ds_consensus of its result in ONE
 * pass over the stacks.
 *
 * Paper: Listing 1 (optimizer.step(), Average(model, group)) and Sec. IV-B2
 * (Lemma 1's left side).  After the step the members of a group hold the
 * group's mean m_k, so with n_k = |g_k|
 *     xbar[p] = (1/W) * sum_k n_k * m_k[p];   dev_out[i] = || m_{g(i)} - xbar ||_2
 * are the consensus norms of the updated stack, and the kernel that takes the
 * step has every m_k in registers: a wavefront owns 256 columns of ALL groups,
 * takes the step group by group, forms xbar in fp64 and sums the squared
 * differences as ds_consensus does (fp32 pair for the mean, fp32 squares, fp64
 * above the lane).  The replica stack is not read a second time: 12 (10 with
 * bf16 gradients) instead of 16 (14) bytes per (worker, column) for step plus
 * norms, and two launches instead of three.  X afterwards is bit for bit what
 * ds_group_sync leaves; dev_out agrees with ds_consensus of it to rounding.
 * When to use it: the pass walks all 2W row streams of the stacks at once, and
 * HBM sustains less over that many streams than over the 2|g| of ds_group_sync
 * (measured 5.3 against 6.4 TB/s at W = 32, groups of 8), so it wins where
 * launches and latency dominate - stacks that fit the last-level cache, e.g.
 * 8 x 1 M parameters: 30 us against 45 us for ds_group_sync + ds_consensus -
 * while on large stacks ds_group_sync followed by ds_consensus_grouped is the
 * faster way to the same norms.
 *
 *   workspace  dev, 16-byte aligned, >= ds_group_sync_consensus_workspace_bytes(P, n_groups)
 *              bytes (one fp64 partial sum per group and tile of 256 columns), overwritten
 *   dev_out    dev fp64 [W], written (zeros if P == 0)
 * Other arguments as ds_group_sync (plain step, fp32 or bf16 gradients).
 * Errors: those of ds_group_sync, DS_ERR_WORKSPACE, DS_ERR_ALIGN for dev_out.
 */
size_t ds_group_sync_consensus_workspace_bytes(int64_t P, int32_t n_groups);

int ds_group_sync_consensus(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx, int64_t ldg,
                            int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups, float lr,
                            double* dev_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tiled stacks -- a second memory layout for the replica, gradient and state
 * stacks, for callers who are free to choose one.
 *
 * Paper: Sec. IV-B2 stacks the replicas as the rows of X_k; how the stack lies
 * in memory is not part of the method.  Element (worker i, column p) of a tiled
 * stack is at
 *     base + (p / 256) * tile_stride + i * 256 + (p % 256)
 * i.e. the W pieces of 256 columns that make up a column tile form one
 * contiguous block of W*256 elements, and the blocks follow each other at
 * tile_stride >= W*256 elements (a multiple of 256).  A stack of P columns has
 * ceil(P/256) blocks (the last one may be partly used: slots that stand for
 * columns at or beyond P, and the space between blocks, are never read or
 * written); the caller owns (ceil(P/256) - 1) * tile_stride + W*256 elements
 * from the base, and ds_tiled_elements is that size rounded up to whole blocks
 * for tile_stride = W*256.  Walked block by block, the step touches two
 * sequential streams whatever the division, instead of one stream per member
 * row: measured on MI355X about 3 % faster than row-major stacks for the step
 * and for the consensus pass alike (W = 16..64 workers, 11.7 M to 138 M
 * columns), 5 to 9 % where the stacks fit the last-level cache; the one-pass
 * step+norms gains the same 3 % and stays behind the plain step there.
 *
 * ds_group_sync_tiled            as ds_group_sync_opt (opt may be NULL); in opt,
 *                                ldv / lds are the tile strides of V and S
 * ds_consensus_tiled             as ds_consensus
 * ds_consensus_grouped_tiled     as ds_consensus_grouped
 * ds_group_sync_consensus_tiled  as ds_group_sync_consensus
 * with tile strides in place of leading dimensions.  Same arithmetic as the
 * row-major entry points: results are bit-identical element for element.
 * Bases 16-byte aligned (fastest: 1-KiB aligned, so that every piece is one
 * aligned KiB).  Errors as the row-major entry points; a tile stride below
 * W*256 is DS_ERR_BAD_SHAPE, one that is not a multiple of 256 DS_ERR_ALIGN;
 * ds_group_sync_tiled covers at most DS_MAX_COLUMNS / n_groups columns per
 * launch (its grid is tiles x groups along x).
 */
#define DS_TILE_COLUMNS 256

int64_t ds_tiled_elements(int64_t P, int32_t W);

int ds_group_sync_tiled(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t tile_stride_x,
                        int64_t tile_stride_g, int32_t W, const int32_t* perm, const int32_t* off,
                        int32_t n_groups, float lr, const ds_local_opt* opt, void* stream);

int ds_consensus_tiled(const void* X, int64_t P, int64_t tile_stride, int32_t W, double* dev_out,
                       void* workspace, size_t workspace_bytes, void* stream);

int ds_consensus_grouped_tiled(const void* X, int64_t P, int64_t tile_stride, int32_t W, const int32_t* perm,
                               const int32_t* off, int32_t n_groups, double* dev_out, void* workspace,
                               size_t workspace_bytes, void* stream);

int ds_group_sync_consensus_tiled(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t tile_stride_x,
                                  int64_t tile_stride_g, int32_t W, const int32_t* perm, const int32_t* off,
                                  int32_t n_groups, float lr, double* dev_out, void* workspace,
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

#ifdef __cplusplus
}
#endif
#endif /* DSSYNC_H */
