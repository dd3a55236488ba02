/*
 * libngc -- nested gradient coding (NGC) on one AMD Instinct MI355X (gfx950).
 *
 * One GPU plays all n workers of the coded distributed gradient descent of
 * Sec. II-C: the data matrix is split into k row blocks (k = n, or k = c*n with
 * c blocks per atomic task), block j yields the partial gradient g_j, worker i sends the linear combination
 * c_i = sum_j B_sigma[i][j] g_j under the component code sigma chosen for this
 * iteration (Sec. III, Defs. 1-2), and the main node recovers the full gradient
 * sum_j g_j = sum_{i in responders} a_i c_i with a decode vector a that
 * satisfies a B_sigma = 1 and vanishes at the stragglers.
 *
 * Conventions
 *  - Every call returns NGC_OK (0) or a negative NGC_ERR_* code; nothing
 *    throws or aborts.  ngc_strerror() names a code, ngc_last_error() gives the
 *    detail of the last failure on a context.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary
 *    host memory.  The caller owns every buffer passed in; the library neither
 *    frees nor keeps them beyond the stream work of the call.  The context owns
 *    only its private workspace (block partials, uploaded code tables).
 *  - Device work is enqueued on the HIP stream given to ngc_create() and is
 *    asynchronous; outputs are fully overwritten, never accumulated into.
 *  - ngc_create, ngc_set_code, ngc_build_code, ngc_get_code, ngc_get_shape,
 *    the ngc_select_* calls, the worker schedule and decoding-table queries,
 *    the closed-form latency calls, ngc_destroy and ngc_strerror touch no
 *    device state and work on a machine without a GPU.
 *  - All matrices are row-major and dense unless stated otherwise.  Device data
 *    is fp32; code matrices and decode vectors are fp64 on the host.
 *  - Calls on one context must not overlap in time from several host threads.
 */
#ifndef NGC_H
#define NGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ngc_ctx ngc_ctx;

enum {
    NGC_OK = 0,
    NGC_ERR_INVALID = -1,     /* bad shape, null pointer, layer out of range, n does not divide k */
    NGC_ERR_UNDECODABLE = -2, /* more stragglers than the largest tolerance s_{L-1}          */
    NGC_ERR_SINGULAR = -3,    /* no a with |a^T B_S - 1| below tolerance (B violates Def. 1) */
    NGC_ERR_HIP = -4,         /* a HIP runtime call failed                                   */
    NGC_ERR_NOMEM = -5,       /* host or device allocation failed                            */
    NGC_ERR_STATE = -6        /* call needs something not yet set (a code layer, MLP shape)  */
};

enum { NGC_LOSS_LSQ = 0, NGC_LOSS_LOGISTIC = 1, NGC_LOSS_MLP2 = 2 };
enum { NGC_CODE_CYCLIC = 0, NGC_CODE_FRACREP = 1 };

/* Kernel ids for ngc_profile_read(). */
enum {
    NGC_KERNEL_GRAD = 0,    /* single-pass partition-gradient kernel (or the two generic passes) */
    NGC_KERNEL_REDUCE = 1,  /* fixed-order sum of block partials                             */
    NGC_KERNEL_ENCODE = 2,
    NGC_KERNEL_DECODE = 3,
    NGC_KERNEL_UPDATE = 4,
    NGC_KERNEL_MLP = 5,     /* all GEMM-shaped kernels of the MLP gradient                  */
    NGC_KERNEL_PROBE = 6,   /* ngc_probe_copy / ngc_probe_read                              */
    NGC_KERNEL_TAIL = 7,    /* fused reduce + encode + decode + update of ngc_iteration     */
    NGC_KERNEL_ROUNDS = 8,  /* fused encode + decode of ngc_encode_decode / ngc_coded_rounds */
    NGC_KERNEL_COUNT = 9
};

/*
 * Create a context for n workers, k partitions and L nested layers
 * (Sec. III, Def. 2).  s[0..L-1] are the straggler tolerances of the layers,
 * strictly ascending with s[0] == 0 and s[L-1] < n; they may be a subset of
 * 0..s_max (a subset of component codes of a nested code is nested).  d is the
 * gradient length (the paper's l).  k = c*n for an integer c >= 1 (Sec. II-C
 * works with k = n and notes that k/n partial gradients can be assigned
 * jointly as one atomic task: worker i then treats the c partitions
 * j*c .. j*c+c-1 of group j like the single partition j), 1 <= n <= k <= 64,
 * 1 <= d <= 2^33.
 * hip_stream is a hipStream_t (NULL = the default stream); it must outlive the
 * context.  Layer 0 is preset to B_0 = I (x) 1_{1 x c} (Alg. 1); the other
 * layers must be given by ngc_set_code() or ngc_build_code() before use.
 * No HIP call is made here.
 */
int ngc_create(ngc_ctx** out, int n, int k, int L, const int* s, int64_t d, void* hip_stream);

/* Release the context and its workspace.  NULL is allowed. */
void ngc_destroy(ngc_ctx* ctx);

/*
 * Install the encoding matrix B_sigma of one layer (Def. 1): B_host is n x k
 * fp64 row-major with zeros outside each row's support.  Rejected with
 * NGC_ERR_INVALID if worker i does not hold its own partition(s) i*c..i*c+c-1
 * (needed for nesting with B_0 = I), or if a row's support does not contain
 * the support of the same row in the layer below (Def. 2, second bullet;
 * checked against layers already set).  The values are copied.
 */
int ngc_set_code(ngc_ctx* ctx, int layer, const double* B_host);

/* Copy the layer's B (n x k fp64 row-major) to B_host_out. */
int ngc_get_code(const ngc_ctx* ctx, int layer, double* B_host_out);

/* The sizes the context was created with (any output pointer may be null), and the
 * input width of the perceptron (0 until ngc_set_mlp2_shape).  For callers and bindings
 * that want to check buffer sizes before handing raw pointers over. */
int ngc_get_shape(const ngc_ctx* ctx, int* n_out, int* k_out, int* layers_out, int64_t* d_out,
                  int* mlp_d_in_out);

/*
 * Build all layers (Alg. 1).  NGC_CODE_CYCLIC: row i of the layer with
 * tolerance sigma is supported on columns {i..i+sigma} mod n (Lemma 2, with the
 * window length sigma+1 that matches the load (k/n)(sigma+1) of Sec. II-C) and
 * lies in the null space of a random sigma x n matrix whose rows sum to zero,
 * so any n-sigma rows span a space containing the all-ones vector (Def. 1);
 * out of several random draws the one that magnifies message rounding least is
 * kept.  NGC_CODE_FRACREP: all-ones rows on blocks of sigma+1 consecutive
 * partitions; needs (s[u]+1) | n and (s[u]+1) | (s[u+1]+1).  For k = c*n the
 * n x n matrix is widened to n x k by repeating each column c times (row
 * weight (k/n)(sigma+1), Def. 1 third bullet).  Random numbers
 * come from a counter-based generator keyed by seed; the same seed gives the
 * same code on every machine.
 */
int ngc_build_code(ngc_ctx* ctx, int kind, uint64_t seed);

/* Shape of the 2-layer perceptron for NGC_LOSS_MLP2: theta is the concatenation
 * [W1 (d_in x hidden) | b1 (hidden) | W2 (hidden x classes) | b2 (classes)] and
 * its length must equal the context's d.  Any d_in and hidden width; at most 16
 * classes (ngc_partition_grads returns NGC_ERR_INVALID beyond that). */
int ngc_set_mlp2_shape(ngc_ctx* ctx, int d_in, int hidden, int classes);

/*
 * Partial gradients of all k row blocks at theta (Sec. II-C):
 *   G[j] = sum over the rows of block j of grad_theta L(y, f(x, theta)),
 * a plain sum (the 1/m of the update rule, Sec. II-B eq. (1), is not applied).
 *   NGC_LOSS_LSQ       L = (x.theta - y)^2 / 2;       y_dev: float [k][rows]
 *   NGC_LOSS_LOGISTIC  L = log(1 + exp(-y x.theta));  y_dev: float +/-1 [k][rows]
 *   NGC_LOSS_MLP2      softmax cross-entropy of relu(x W1 + b1) W2 + b2;
 *                      y_dev: int32 class ids [k][rows]
 * X_dev: float [k][rows_per_part][d_in] row-major (d_in = d for the first two
 * losses), 16-byte aligned.  theta_dev: float [d].  G_dev: float [k][d], fully
 * overwritten.  Each row of X is read from HBM exactly once for every
 * d <= 32768 that is a multiple of 4 and every d <= 16384 that is not (fastest
 * when d is 256, 512, 768 or a multiple of 1024); larger d take a two-pass
 * route that reads X twice.
 * Accumulation is fp32 with a fixed summation order (bit-reproducible).
 */
int ngc_partition_grads(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                        const float* theta_dev, int64_t rows_per_part, float* G_dev);

/*
 * ngc_partition_grads for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and, for a shape it accepts, the same bits as ngc_partition_grads, but the block
 * partials of the gradient kernels go to a device array of fixed size that is part of the
 * library image (20 MiB, held by every GPU the library runs on until the process ends)
 * instead of the context's workspace.  The call makes no hipMalloc / hipFree and creates no
 * event (its launches are not recorded by ngc_profile_*).  The very first call on a device
 * looks up the array's address there; make that call outside a capture.
 *   Limits: NGC_LOSS_LSQ and NGC_LOSS_LOGISTIC only (the perceptron's activations do not
 *   fit), and shapes whose block partials fit the array: every single-pass shape with
 *   d <= 16384 does, wider single-pass rows (one block per compute unit, 4 d bytes each)
 *   up to d = 20480 on a GPU of 256 compute units; for the two-pass shapes
 *   4 * k * (d + rows_per_part) bytes plus 0.5 MiB must stay below 20 MiB.  Anything else returns NGC_ERR_INVALID and launches nothing.
 *   All calls on one GPU share the one array, whichever context they use: calls that
 *   overlap in time on one GPU (two streams, two host threads) race on it.  Nothing in it
 *   has to start at zero (every partial is written before it is read), so it is not cleared.
 */
int ngc_partition_grads_static(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                               const float* theta_dev, int64_t rows_per_part, float* G_dev);

/*
 * Worker messages C = B G (Sec. II-C) layer by layer:
 *   C[u][i][:] = sum_j B^(u)[i][j] G[j][:]   in fp32.
 * G_dev: float [k][d].  C_dev: float [L][n][d].  layer = -1 encodes every
 * layer in one pass over G; layer = u writes only slice u of C_dev.
 */
int ngc_encode(ngc_ctx* ctx, const float* G_dev, int layer, float* C_dev);

/*
 * Main-node bookkeeping for one iteration, on the host.
 * straggler_mask[i] != 0 marks worker i as a straggler.  The layer chosen is
 * the smallest u with s[u] >= number of stragglers (Observation after Def. 2);
 * NGC_ERR_UNDECODABLE if there is none.  a_out[n] receives the least-2-norm
 * solution of a^T B^(u) = 1^T with a_i = 0 at every straggler (a row of A_sigma
 * in the sense of Def. 1: supported on responders, a B = 1; when exactly
 * n - s[u] workers respond it is the only one).  residual_out (may be NULL)
 * receives max_j |(a^T B)_j - 1|; above 1e-6 the call returns
 * NGC_ERR_SINGULAR.  layer_out is written even when that happens.
 */
int ngc_select_decode_vec(const ngc_ctx* ctx, const uint8_t* straggler_mask, int* layer_out,
                          double* a_out, double* residual_out);

/*
 * Guarded layer choice (an option; off by default, and then the rule above holds as stated).
 * Every component code with s[v] >= number of stragglers recovers the gradient (Def. 1), and a
 * main node whose responders hold the messages of all their layers may take a larger one.
 * With exactly s[u] stragglers the layer-u decode vector is the only one there is, and for a
 * real-valued code it can be large enough to lift the rounding of fp32 messages above a
 * tolerance.  With a limit set, ngc_select_decode_vec, ngc_coded_rounds and ngc_iteration
 * estimate that amplification for the vector they find,
 *   kappa_hat = sum_i |a_i| ||b_i||_2 / sqrt(k)
 * (the factor for partial gradients with independent entries of equal variance; the decoded
 * gradient is then off by about 0.1 * 2^-24 * kappa_hat in relative 2-norm, 4 * 2^-24 *
 * kappa_hat at most), and if it exceeds the limit move up to the first layer whose estimate is
 * within it, or to the layer of smallest estimate if none is (the lowest of them on a tie).
 * kappa_limit > 0 sets the limit; 0 or +infinity switches the guard off; negative or NaN is
 * NGC_ERR_INVALID.  Not applied by ngc_select_decode_vec_first, ngc_select_from_progress
 * (workers there have not computed the larger layers) or ngc_decode_lookup.
 */
int ngc_set_decode_guard(ngc_ctx* ctx, double kappa_limit);

/*
 * Same bookkeeping with the decode vector supported on the n - s[u]
 * responders of lowest index only (a literal row of the decoding matrix of
 * Def. 1).
 */
int ngc_select_decode_vec_first(const ngc_ctx* ctx, const uint8_t* straggler_mask,
                                int* layer_out, double* a_out, double* residual_out);

/*
 * Main-node recovery (Def. 1, A B = 1):  g[:] = sum_i a[i] * C[layer][i][:]
 * over the workers with a[i] != 0.  a_host: double [n] (read before the call
 * returns).  C_dev: float [L][n][d] as written by ngc_encode.  g_dev: float [d].
 * Products and the sum are formed in fp64 and rounded once to fp32.
 */
int ngc_decode(ngc_ctx* ctx, int layer, const double* a_host, const float* C_dev, float* g_dev);

/*
 * Encode and decode of one round in one pass over G (Sec. II-C, X = B G, followed by the
 * recovery of Def. 1): for every worker i with a[i] != 0 the message of the given layer
 *   M[i][:] = fp32( sum_j B^(layer)[i][j] G[j][:] )
 * is formed, rounded to fp32 and written (a worker sends fp32; rows of stragglers are left
 * untouched), and  g[:] = fp32( sum_i a[i] * (double) M[i][:] )  is accumulated from the
 * rounded messages while they are still in registers: G is read once, no message is read
 * back.  Same bits as ngc_encode(layer) followed by ngc_decode(layer, a) on the rows it
 * writes.  G_dev: float [k][d].  a_host: double [n], as returned by ngc_select_decode_vec.
 * M_dev: float [n][d].  g_dev: float [d].  Asynchronous on the context's stream.
 */
int ngc_encode_decode(ngc_ctx* ctx, const float* G_dev, int layer, const double* a_host,
                      float* M_dev, float* g_dev);

/*
 * Many rounds of encode + decode per launch.  masks_host: uint8 [rounds][n], one
 * straggler mask per round (1 = straggler).  For every round r the main node's bookkeeping
 * (layer by the Observation after Def. 2, least-norm decode vector as in
 * ngc_select_decode_vec) is done on the host, the vectors go to the device as a table, and a
 * kernel forms, for every round of its run, the messages of that round's layer for its
 * responders and the recovered gradient, exactly as ngc_encode_decode does (same bits).  Up
 * to 255 rounds are one run; more go as a first run of 64 (so that the device starts early)
 * and runs of 256 after it, one launch each, the host solving for the next run while the
 * device works on the current one; a run's table travels on a stream of the library's own
 * and its kernel, on the context's stream, waits for it:
 *   G of round r  = G_dev + r * g_round_stride   (float [k][d]; stride 0: one G for all rounds,
 *                                                 read from HBM once per block, else >= k*d)
 *   messages      -> M_dev + r * m_round_stride  (float [n][d]; stride >= n*d)
 *   gradient      -> g_dev + r * d               (float [rounds][d])
 * layers_out (int [rounds], may be NULL) receives each round's layer, -1 for a round with
 * more stragglers than the largest tolerance: such a round writes a zero gradient and no
 * message and is not an error.  a_out (double [rounds][n], may be NULL) receives the decode
 * vectors.  NGC_ERR_SINGULAR if a round's residual is above tolerance: the run that holds the
 * round and the runs after it are not launched (earlier runs are).  The host part uses a few
 * threads, kept by the context between calls, when the solves are worth them; the call
 * returns when the last kernel is enqueued.  Not for use under stream capture.
 */
int ngc_coded_rounds(ngc_ctx* ctx, const float* G_dev, int64_t g_round_stride, int rounds,
                     const uint8_t* masks_host, float* M_dev, int64_t m_round_stride, float* g_dev,
                     int* layers_out, double* a_out);

/*
 * Redundancy-faithful execution (Sec. III, layered task scheduling): worker i
 * works through the partitions of its nested supports layer by layer -- its own
 * partition first (sigma = 0), then what each larger sigma adds, new partitions
 * of a layer in cyclic order from index i -- and computes every partial gradient
 * itself, so a partition held by s+1 workers is read s+1 times.
 *
 * ngc_worker_task_count: length T of the longest schedule in atomic tasks of
 *   c = k/n partitions (s_max + 1 for the codes built here).
 *   ngc_worker_schedule: the partitions of one worker in the order it works
 *   through them, c per task (parts_out has room for T*c entries).
 * ngc_worker_grads: progress_host[i] = number of tasks worker i has finished
 *   (0..T).  W_dev: float [n][T*c][d]; row (i, t) receives the partial gradient
 *   of the t-th partition of worker i's schedule for t < c*progress[i]; other
 *   rows are left untouched.  All three losses (the perceptron after
 *   ngc_set_mlp2_shape; its units run as one batched launch per stage).
 * ngc_worker_encode: C[u][i][:] = sum_t B^(u)[i][part(i,t)] W[i][t][:] (Sec.
 *   II-C, X = B G, from the worker's own copies) for every layer u whose
 *   s[u]+1 tasks worker i has finished; rows of unfinished (u, i) are set to
 *   zero.  C_dev: float [L][n][d].  Any number of layers (Def. 2: sigma = 0..s_max);
 *   a worker's rows of W are read once per run of eight layers.  Only rows the worker
 *   has computed are read (at most its own schedule's length).
 * ngc_select_from_progress: the main node's termination rule (Sec. IV, proof of
 *   Theorem 1): the smallest layer u >= min_layer for which at least n - s[u]
 *   workers have finished their layer-u tasks; mask_out[i] = 1 for workers not
 *   among them; a_out = least-norm decode vector over those that are.
 *   NGC_ERR_UNDECODABLE if no layer qualifies yet.  min_layer = index of sigma
 *   restricts the scheme to a conventional gradient code with that fixed
 *   sigma (Def. 1).  Host only.
 */
int ngc_worker_task_count(const ngc_ctx* ctx, int* tasks_out);
int ngc_worker_schedule(const ngc_ctx* ctx, int worker, int* parts_out, int* count_out);
int ngc_worker_grads(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev,
                     const float* theta_dev, int64_t rows_per_part, const int* progress_host,
                     float* W_dev);
int ngc_worker_encode(ngc_ctx* ctx, const float* W_dev, const int* progress_host, float* C_dev);
int ngc_select_from_progress(const ngc_ctx* ctx, const int* progress_host, int min_layer,
                             int* layer_out, uint8_t* mask_out, double* a_out,
                             double* residual_out);

/*
 * Latency model (Secs. II-D and IV).  A non-failing worker finishes u tasks at
 * gamma + eps + u*rho + Erlang(u, lambda) (eq. (2)); it fails for good with
 * probability pe.  1 <= n <= 64, 0 <= sigma, smax < n, lambda > 0, the other
 * parameters >= 0, pe <= 1.
 *
 * ngc_latency_cdf_gc: P(T_GC <= t[q]) of a conventional (n,k,sigma) gradient
 *   code (Lemma 1).  ngc_latency_cdf_ngc: P(T_NGC <= t[q]) of an (n,k,smax)
 *   nested code with component codes sigma = 0..smax (Theorem 1, summation
 *   limits as in its proof: a configuration is undecodable when at every layer
 *   u fewer than n-u+1 workers have finished u tasks).  t and cdf_out are host
 *   arrays of nt entries.  Host only.
 * ngc_latency_simulate: Monte-Carlo draws of the same model on the device,
 *   one wave per trial.  L_dev: double [smax+1][trials]; L[u-1][r] = time at
 *   which n-u+1 workers have finished u tasks in trial r (+inf if never), so
 *   the conventional code with tolerance sigma has latency L[sigma][r].
 *   Tngc_dev (may be NULL): double [trials], min_u L[u-1][r], the nested
 *   code's latency.  Random numbers: Philox-4x32-10 with key = seed and
 *   counter = (trial, worker, block, 0); word 0 of a worker decides failure
 *   (U < pe), word u is its u-th task time rho - log(U)/lambda,
 *   U = (word + 0.5)/2^32.  trials < 2^32.  hip_stream: hipStream_t or NULL.
 */
int ngc_latency_cdf_gc(int n, int sigma, double lambda, double rho, double eps, double gamma,
                       double pe, const double* t, int nt, double* cdf_out);
int ngc_latency_cdf_ngc(int n, int smax, double lambda, double rho, double eps, double gamma,
                        double pe, const double* t, int nt, double* cdf_out);
int ngc_latency_simulate(void* hip_stream, int n, int smax, double lambda, double rho, double eps,
                         double gamma, double pe, uint64_t seed, int64_t trials, double* L_dev,
                         double* Tngc_dev);

/*
 * Explicit decoding matrix A_sigma of one layer (Def. 1, first, fourth and
 * fifth bullet): one row per straggler set of size sigma = s[layer], in
 * lexicographic order of the sorted sets; row j is supported on the n - sigma
 * responders of its set and satisfies a_j B_sigma = 1.  Only for small codes:
 * refused above 2^20 rows.
 *
 * ngc_build_decoding_table: build (or rebuild) the table on the host; rows_out
 *   (may be NULL) receives C(n, sigma).  Installing a new B for the layer
 *   discards the table.
 * ngc_decoding_row_index: row that serves a straggler mask.  With fewer than
 *   sigma stragglers the responders of highest index are left unused, i.e.
 *   the n - sigma responders of lowest index decode.  More than sigma
 *   stragglers: NGC_ERR_UNDECODABLE.
 * ngc_get_decoding_row: copy one row (n doubles) to a_out.
 * ngc_decode_lookup: ngc_decode with the decode vector read by the kernel from
 *   the table's device copy (uploaded on first use); the host only ranks the
 *   mask, no system is solved per iteration.
 */
int ngc_build_decoding_table(ngc_ctx* ctx, int layer, int64_t* rows_out);
int ngc_decoding_row_index(const ngc_ctx* ctx, int layer, const uint8_t* straggler_mask,
                           int64_t* row_out);
int ngc_get_decoding_row(const ngc_ctx* ctx, int layer, int64_t row, double* a_out);
int ngc_decode_lookup(ngc_ctx* ctx, int layer, const uint8_t* straggler_mask, const float* C_dev,
                      float* g_dev);

/* theta[:] -= scale * g[:]  with scale = eta/m  (Sec. II-B eq. (1)). */
int ngc_update(ngc_ctx* ctx, float* theta_dev, const float* g_dev, double scale);

/*
 * One whole iteration (Sec. II-C; update of Sec. II-B eq. (1)): partition
 * gradients at theta, messages of every layer, layer and least-norm decode
 * vector for the straggler mask, decode, theta <- theta - scale * g.  Same
 * results, bit for bit, as ngc_partition_grads, ngc_encode(-1),
 * ngc_select_decode_vec, ngc_decode, ngc_update in sequence, but for the two
 * regression losses everything after the gradient kernel is one launch that
 * reads that kernel's block partials column tile by column tile.  G_dev
 * [k][d], C_dev [L][n][d], g_dev [d] are all written; theta_dev is read and
 * updated; all five device buffers 16-byte aligned.  layer_out / a_out (n
 * doubles) may be NULL.  An undecodable mask returns NGC_ERR_UNDECODABLE before
 * anything is launched (theta stays as it is).  The second launch keeps its column
 * tiles, and the compressed code tables if they fit beside them, in LDS; tables too
 * large for that (the full layer set sigma = 0..31 of 64 workers has 33 792 non-zeros)
 * are read from global memory instead, with the same results.
 */
int ngc_iteration(ngc_ctx* ctx, int loss, const float* X_dev, const void* y_dev, float* theta_dev,
                  int64_t rows_per_part, const uint8_t* straggler_mask, double scale, float* G_dev,
                  float* C_dev, float* g_dev, int* layer_out, double* a_out);

/* LDS bytes per block of ngc_iteration's second launch at vector width 1, 2 or 4 floats per
 * lane, with the code tables in LDS and without (either output may be NULL).  Host only;
 * every layer must have its code. */
int ngc_tail_lds_bytes(const ngc_ctx* ctx, int vec_width, int64_t* with_tables_out,
                       int64_t* without_tables_out);

/* Block until the context's stream is idle. */
int ngc_sync(ngc_ctx* ctx);

/*
 * Per-kernel timing.  kernel_mask selects the kernel ids to time (bit k =
 * NGC_KERNEL_k, -1 = all, 0 = off); each launch of a selected kernel is
 * bracketed by HIP events on the context's stream.  ngc_profile_read()
 * synchronises, adds the elapsed times up per kernel id, writes launch counts
 * and total milliseconds (arrays of NGC_KERNEL_COUNT) and clears the record.
 * At most 4096 launches are recorded between reads; later ones run untimed.
 */
int ngc_profile_enable(ngc_ctx* ctx, int kernel_mask);
int ngc_profile_read(ngc_ctx* ctx, int64_t* launches_out, double* total_ms_out);
/*
 * The recorded launches of one kernel id one by one, in launch order:
 * synchronises, writes up to `capacity` durations in milliseconds to ms_out
 * (host) and the number of recorded launches of that kernel to count_out.  The
 * record is left as it is; call before ngc_profile_read(), which clears it.
 */
int ngc_profile_launches(ngc_ctx* ctx, int kernel, double* ms_out, int64_t capacity,
                         int64_t* count_out);

/*
 * Measurement aids, not part of the method.  ngc_probe_copy copies `bytes`
 * (a multiple of 16, both pointers 16-byte aligned, buffers must not overlap)
 * with a plain kernel: a dispatch of known HBM traffic against which byte
 * counters can be calibrated.  ngc_probe_read streams `bytes` once through a
 * plain read-and-add kernel: the read bandwidth a trivial kernel reaches.
 * Both are recorded under NGC_KERNEL_PROBE when profiling is on.
 */
int ngc_probe_copy(ngc_ctx* ctx, const void* src_dev, void* dst_dev, int64_t bytes);
int ngc_probe_read(ngc_ctx* ctx, const void* src_dev, int64_t bytes);

const char* ngc_strerror(int code);
const char* ngc_last_error(const ngc_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* NGC_H */
