/*
 * libsom — batch self-organising-map training epoch on one AMD MI355X (gfx950).
 *
 * C ABI, plain pointers and sizes.  Every pointer argument is marked [device] (memory of the context's GPU,
 * e.g. obtained from hipMalloc or a torch tensor's data_ptr) or [host].  All matrices are row-major.
 *
 * Notation (the paper's, Section 3.3.1):
 *   X      N x D samples, float32, leading dimension ldx >= D (in floats); may be NULL when N == 0
 *   idx    optional list of m presented row numbers into X (Section 3.1, Eq. 2: the iteration subset);
 *          NULL means rows 0..N-1 are presented and m must equal N
 *   W      K x D node weights, float32, dense (leading dimension D)
 *   b(x)   best-matching unit of x: argmin_k |x - w_k|^2 under the weights at the start of the epoch,
 *          lowest node index among exact float32 minima
 *   S_k    sum of the presented samples whose BMU is k;  n_k their count
 *   G      K x K neighbourhood distances between nodes, float32: G[k*K + j] is the distance from BMU node k
 *          to updated node j (lattice distance for grid / hexagonal maps, graph hop count for the MST and
 *          RNG topologies of Sections 3.2.1-3.2.2; +inf = no influence)
 *   sigma  neighbourhood radius of this epoch;  h(g) = exp(-g^2 / (2 sigma^2))
 *
 * One epoch (Eq. 3 with learning rate 1 and no momentum; the new weight is the ratio U_j / H_j of the paragraph
 * after Eq. 4, guarded where H_j vanishes):
 *   Num_j = sum_k h(G[k][j]) S_k,   Den_j = sum_k h(G[k][j]) n_k,
 *   w_j  <- Num_j / Den_j   if Den_j >= eps_h,   otherwise w_j is left unchanged.
 * Grouping the per-sample sums of Eq. 3 by BMU gives exactly this form.
 *
 * Calls return SOM_OK or a negative code; they never abort and never throw.  Arguments are checked first and
 * a rejected call has no side effects.  Work is enqueued on the context's stream and the call returns without
 * waiting, unless a [host] output is requested (som_epoch's stats, som_epoch_host, som_epoch_file).  The caller owns every
 * buffer it passes and keeps it alive until som_sync (or a synchronising call) returns; the library owns only
 * its internal workspaces.  A context is bound to one device and is not thread-safe.
 */
#ifndef SOM_H
#define SOM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct som_ctx som_ctx;

enum {
    SOM_OK = 0,
    SOM_EINVAL = -1, /* bad argument (null pointer, non-positive size, ldx < D, m != N without idx, ...) */
    SOM_ENOMEM = -2, /* a workspace allocation failed */
    SOM_EHIP = -3,   /* a HIP runtime call or kernel launch failed; see som_last_error */
    SOM_EIO = -4,    /* som_epoch_file: the sample file is too short or a read failed; see som_last_error */
    SOM_ESTATE = -5  /* context unusable (no gfx950 device, destroyed) */
};

enum { SOM_KERNEL_GAUSSIAN = 0 /* h(g) = exp(-g^2 / (2 sigma^2)) */ };

enum {
    SOM_TOPOLOGY_MST = 1, /* minimum spanning tree over the node weights (Algorithm 1) */
    SOM_TOPOLOGY_RNG = 2  /* relative neighbourhood graph (Algorithm 2) */
};

/* Create a context on HIP device `device`.  `hip_stream` is the hipStream_t the library enqueues all compute on
 * (e.g. the caller's torch stream); NULL is HIP's default stream.  The stream stays the caller's.  The library
 * creates one further stream of its own for host-to-device copies.  *out receives the context. */
int som_create(som_ctx** out, int device, void* hip_stream);
void som_destroy(som_ctx* ctx);
/* Static description of a return code. */
const char* som_strerror(int code);
/* Detail of the last failure on this context (owned by the context, valid until the next call). */
const char* som_last_error(const som_ctx* ctx);
/* Block until everything enqueued on the context's stream has finished. */
int som_sync(som_ctx* ctx);

/*
 * Measurement support (not an operation of the paper).  While profiling is enabled the library brackets every
 * launch of its BMU search kernel (in the default search together with the small kernel that compacts the
 * search's per-sample marks into the re-decision list) with a pair of HIP events on the context's stream; som_profile_read waits for the
 * stream, writes up to `capacity` kernel durations in milliseconds (launch order) to ms [host], stores the number
 * of launches recorded since the last read in *count [host], and starts a new record.  A call over more rows than one
 * pass holds (2^27; fewer for D > 64 in the default search, whose pass must fit the samples' bf16 parts into 8 GB)
 * launches the kernel once per pass; for D > 64 in the default search a launch's bracket includes the conversion of
 * the pass's samples.
 */
int som_profile(som_ctx* ctx, int enable);
int som_profile_read(som_ctx* ctx, float* ms, int32_t capacity, int32_t* count);

/*
 * Measurement support (not an operation of the paper): the accumulation behaviour of the bf16 matrix pipe, on which
 * the rounding bound of the default search rests.  For each of n problems one v_mfma_f32_32x32x16_bf16 is executed:
 *     Dout[t][i][j] = C[t][i][j] + sum_{k < 16} A[t][i][k] * Bt[t][j][k]
 *   A, Bt [device] uint16[n][32][16]: bf16 bit patterns (Bt holds B transposed), 16-byte aligned
 *   C, Dout [device] float[n][32][32]
 * The products are exact in float32; how the pipe adds the seventeen terms is what a caller measures by comparing
 * Dout with the exact sum.  Asynchronous on the context's stream; n <= 2^24.
 */
int som_matrix_pipe_probe(som_ctx* ctx, const uint16_t* A, const uint16_t* Bt, const float* C, float* Dout, int64_t n);

/*
 * Measurement support (not an operation of the paper): a loop of v_mfma_f32_32x32x16_bf16 on pseudo-random operands,
 * eight per trip on two accumulators, with fold_steps (0..2) fold steps of three vector instructions beside each, on one
 * workgroup of four wavefronts per compute unit and waves_per_simd (1 or 2) of them resident.  It executes
 * 8 * iters MFMAs per wavefront; timed by the caller over a second or more it gives the MFMA rate the chip sustains under
 * its power limit for that instruction mix, the practical ceiling of the default BMU search's stage loop.
 */
int som_mfma_rate_probe(som_ctx* ctx, int fold_steps, int waves_per_simd, int iters);

/*
 * Measurement support (not an operation of the paper): one plain streaming read of `bytes` bytes at p [device] (16-byte
 * loads, nothing else), enqueued on the context's stream.  Timed by the caller, it gives the read bandwidth the memory
 * system delivers to a kernel on this GPU, the yardstick for the HBM-bound accumulation pass.  p and bytes must be
 * multiples of 16.
 */
int som_read_probe(som_ctx* ctx, const void* p, int64_t bytes);

/*
 * Best-matching-unit search (Section 3.3.1, definition of b(x)).
 *   X [device] N x D, ldx;  idx [device] m row numbers or NULL;  W [device] K x D
 *   bmu [device] int32[m], required: bmu[i] = b(x_{idx[i]})
 *   d2  [device] float[m] or NULL: squared distance to the BMU by float32 direct differences: on the values as
 *       given for re-decided samples, on values centred by the column means of W for the others (relative
 *       error up to 6e-5 from the two centring roundings; samples that close to their node are re-decided)
 *   qe  [device] double[2] or NULL, OVERWRITTEN with { sum_i sqrt(d2_i), sum_i d2_i }  (the quantisation
 *       error of Section 4.1.2 is qe[0] / m)
 * The N x K distance matrix is never formed in memory.  m == 0 is allowed (qe becomes {0, 0}).
 * With d2 and qe both NULL no distance is formed for samples that are not re-decided: for 4 <= D <= 64 the default
 * search then reads every row once instead of twice.
 */
int som_bmu(som_ctx* ctx, const float* X, int64_t N, int32_t D, int64_t ldx,
            const uint32_t* idx, int64_t m, const float* W, int32_t K,
            int32_t* bmu, float* d2, double* qe);

/*
 * Per-BMU sums and counts (the inner sums of Eq. 3 grouped by BMU; adding the results of several calls, or of
 * several devices, is Eq. 4).
 *   bmu [device] int32[m], every entry in [0, K)  (entries outside are skipped)
 *   S [device] double[K*D], n [device] uint64[K]: S_k += x, n_k += 1.  zero_first != 0 clears S and n first;
 *   otherwise the call accumulates onto their current contents (chunk-wise accumulation).
 */
int som_accumulate(som_ctx* ctx, const float* X, int64_t N, int32_t D, int64_t ldx,
                   const uint32_t* idx, int64_t m, const int32_t* bmu, int32_t K,
                   double* S, uint64_t* n, int zero_first);

/*
 * Neighbourhood-weighted update (the normalised update U_j / H_j after Eq. 4).
 *   S [device] double[K*D], n [device] uint64[K], G [device] float[K*K]
 *   W [device] K x D float, updated IN PLACE: w_j <- Num_j / Den_j where Den_j >= eps_h, else unchanged
 *   eps_h <= 0 selects the default 1e-30;  kernel must be SOM_KERNEL_GAUSSIAN;  sigma > 0 and finite
 *   n_guarded [device] int32 or NULL: OVERWRITTEN with the number of nodes left unchanged
 * Computed in float64.
 */
int som_neighborhood_update(som_ctx* ctx, const double* S, const uint64_t* n, const float* G,
                            int32_t K, int32_t D, double sigma, int kernel, double eps_h,
                            float* W, int32_t* n_guarded);

/*
 * som_neighborhood_update for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same results as som_neighborhood_update,
 * but the split-k partial sums (and the exponent shifts of SOM_SAFEGUARD_SHIFT) go to a fixed device array of 8.25 MiB
 * that the library holds on each GPU it runs on until the process ends, instead of a workspace grown on demand; the
 * call makes no hipMalloc / hipFree and enqueues no memset (counters are cleared by a small kernel).
 * Limits: D <= 63, K <= 32768 and K * (D + 1) <= 65536 (for instance 1024 nodes x 63 features, 4096 x 15); larger
 * shapes return SOM_EINVAL with the limits in som_last_error and touch nothing.
 * Every call on a GPU, from whatever context or stream, shares that GPU's array: calls that overlap in time on one
 * GPU race and give wrong results; calls ordered on one stream (or otherwise serialised) are safe.
 */
int som_neighborhood_update_static(som_ctx* ctx, const double* S, const uint64_t* n, const float* G,
                                   int32_t K, int32_t D, double sigma, int kernel, double eps_h,
                                   float* W, int32_t* n_guarded);

/*
 * General update rule of the paragraph after Eq. 4: learning rate eta (the eta_t inside U_j of Eq. 3) and
 * optional momentum.  With   u_j = eta (Num_j / Den_j - w_j)   (= U_j / H_j; 0 where Den_j < eps_h)   every
 * later update on this context (som_neighborhood_update, som_epoch, som_epoch_host) applies
 *     delta_j = u_j + mu * velocity_j,    w_j <- w_j + delta_j,    velocity_j <- delta_j.
 * velocity [device] float[K*D], caller-owned, read and written by every update; required when mu != 0, may be
 * NULL otherwise.  eta = 1, mu = 0 (the default of a new context) is the plain rule w_j <- Num_j / Den_j.
 * eta must be in (0, 1], mu in [0, 1).
 */
int som_set_update_rule(som_ctx* ctx, double eta, double mu, float* velocity);

/*
 * Rebuild a data-driven neighbourhood graph from the current weights and return its hop counts
 * (Sections 3.2.1-3.2.2, Algorithms 1 and 2): pairwise squared Euclidean distances between the node weight
 * vectors, then either the minimum spanning tree of the complete graph under those distances, or the relative
 * neighbourhood graph (p ~ q unless a third node r has max(d(p,r), d(q,r)) < d(p,q), strict), then the number
 * of edges on the shortest path between every two nodes.
 *   W [device] K x D float (read only)
 *   kind  SOM_TOPOLOGY_MST or SOM_TOPOLOGY_RNG
 *   G [device] float[K*K], caller-owned, OVERWRITTEN: G[p*K+q] = hop count, 0 on the diagonal, +inf between
 *     nodes in different components (possible only when distances are non-finite)
 * Distances and every comparison that decides an edge are float64 on direct differences.  When several edges
 * have exactly equal length the spanning tree is a minimal one: for K <= 4096 the one that visiting edges in
 * (length, lower end, higher end) order would build, above that the one Prim's method grows from node 0.
 * Asynchronous on the context's stream; K is limited to 12000 by the graph kernels' LDS use.
 */
int som_topology(som_ctx* ctx, const float* W, int32_t K, int32_t D, int kind, float* G);

/*
 * How the update keeps U_j / H_j finite (the paragraph after Eq. 4 asks for a guard and names none), for every later
 * update on this context:
 *   SOM_SAFEGUARD_THRESHOLD (default)  w_j is left unchanged where Den_j < eps_h;
 *   SOM_SAFEGUARD_SHIFT                the exponents of updated node j are shifted by m_j = min over occupied nodes k
 *                                      (n_k > 0) of G[k][j]^2:  h'_kj = exp(-(G[k][j]^2 - m_j) / (2 sigma^2)) for
 *                                      n_k > 0, else 0.  The ratio Num_j / Den_j is the same wherever the plain sums
 *                                      do not underflow; where they do, node j follows its nearest occupied nodes.
 *                                      Nodes no occupied node reaches (m_j infinite) are left unchanged and counted
 *                                      as guarded.
 */
enum { SOM_SAFEGUARD_THRESHOLD = 0, SOM_SAFEGUARD_SHIFT = 1 };
int som_set_safeguard(som_ctx* ctx, int mode);

/*
 * Accumulation order (not an operation of the paper).  By default the per-BMU sums are taken with float64 LDS
 * atomics: counts are exact, a sum can differ between two runs by a few units in its 16th digit because the order
 * of the additions is not fixed.  With on != 0 every later som_accumulate / som_epoch / som_epoch_host on this
 * context uses the slower kernel that adds in a fixed order wherever it applies (K <= 1024, or K <= 2048 with
 * D <= 31): S, and with it W, is then bit-identical from run to run.
 */
int som_set_reproducible(som_ctx* ctx, int on);

/*
 * Which matrix pipe forms the scores of the best-matching-unit search (Section 3.3.1: b(x); not an operation of
 * the paper).  The results are the same either way: every sample whose best two scores lie inside the worst-case
 * rounding bound of the arithmetic in use is re-decided by direct float32 differences.
 *   SOM_SEARCH_AUTO (default)  for D >= 4 and K > 1 the samples and weights are cut into two bf16 parts each
 *                              and a score is the sum of three bf16 MFMA products (worst-case error of a
 *                              difference of two scores: below 2^-14 of |x||w| + |w|^2/2); for D > 64 the samples' parts
 *                              are written once per call into a library-owned workspace of up to 8 GB (rows go
 *                              through in passes that fit it); other shapes use the float32 MFMA search;
 *   SOM_SEARCH_FLOAT32         float32 MFMA for every shape.
 * Applies to every later som_bmu / som_epoch / som_epoch_host on this context.
 */
enum { SOM_SEARCH_AUTO = 0, SOM_SEARCH_FLOAT32 = 1 };
int som_set_search(som_ctx* ctx, int mode);

/* [host] statistics of one epoch, filled after the epoch's work has finished. */
typedef struct {
    double sum_dist;   /* sum over presented samples of the distance to the BMU (pre-update weights) */
    double sum_dist2;  /* same with squared distances */
    int64_t m;         /* samples presented */
    int64_t n_recheck; /* samples whose best two float32 scores were too close and were re-decided exactly */
    int32_t n_empty;   /* nodes that were nobody's BMU */
    int32_t n_guarded; /* nodes left unchanged by the denominator threshold */
    float ms_bmu_acc;  /* device time of BMU + accumulation (all chunks), milliseconds */
    float ms_update;   /* device time of the neighbourhood update */
    float ms_h2d;      /* som_epoch_host: time the copy stream spent on host-to-device transfers */
} som_stats;

/*
 * One whole epoch on device-resident samples: best-matching-unit search over the presented rows (the BMU indices go
 * to a library-owned buffer), per-BMU accumulation in a second pass over the same rows, then the neighbourhood update
 * of W in place.  Arguments as above.  stats is [host] or NULL; a non-NULL stats makes the call wait for the epoch
 * to finish, and only then are the distances to the BMUs and their sums formed at all (they are statistics of the
 * epoch, Section 4.1.2, not part of the update of Eq. 3-4).  m == 0 leaves W unchanged.
 */
int som_epoch(som_ctx* ctx, const float* X, int64_t N, int32_t D, int64_t ldx,
              const uint32_t* idx, int64_t m, float* W, int32_t K,
              const float* G, double sigma, int kernel, double eps_h, som_stats* stats);

/*
 * One whole epoch on samples in HOST memory (Section 3.3.2's chunked loading path: pinned host chunk, copy
 * to the GPU on a side stream overlapped with compute on the previous chunk, accumulators carried across the
 * chunks, one update at the end).  Xhost [host] is any readable N x D float32 array, dense (ldx = D), for
 * instance a memory-mapped file; the library reads all N * D floats of it with memcpy, so a mapping shorter than that
 * faults as any read beyond it would (use som_epoch_file to have a short file reported instead).  chunk_rows > 0 is
 * the chunk length in rows; the library owns two pinned staging buffers and two device buffers of chunk_rows x D
 * floats, allocated on first use and kept until som_destroy.  pinned != 0 promises that Xhost itself is pinned
 * (hipHostMalloc) memory, in which case it is copied from directly.  Always waits for the epoch to finish; after a
 * failure both of the library's streams have been drained and the context stays usable (W is unchanged unless the
 * failure came from the update itself).
 */
int som_epoch_host(som_ctx* ctx, const float* Xhost, int64_t N, int32_t D, int64_t chunk_rows, int pinned,
                   float* W, int32_t K, const float* G, double sigma, int kernel, double eps_h,
                   som_stats* stats);

/*
 * The same epoch on samples in a FILE (the disk-backed regime of Section 3.3.2): rows 0..N-1 are the N * D float32
 * values that start at byte `offset` of the open file descriptor fd (dense, row-major).  Each chunk is read with
 * pread by several host threads straight into a pinned staging buffer (no mapping, no intermediate copy) while the
 * previous chunk is on the GPU.  A regular file shorter than offset + N * D * 4 bytes is rejected up front with
 * SOM_EIO and no side effects; a read error or an early end of file during the epoch returns SOM_EIO after both
 * streams have been drained, W unchanged.  The descriptor stays the caller's; its file position is not used.
 */
int som_epoch_file(som_ctx* ctx, int fd, int64_t offset, int64_t N, int32_t D, int64_t chunk_rows,
                   float* W, int32_t K, const float* G, double sigma, int kernel, double eps_h,
                   som_stats* stats);

#ifdef __cplusplus
}
#endif
#endif /* SOM_H */
