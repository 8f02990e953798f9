/*
 * decentlam.h -- C ABI of the MI355X (gfx950) library for the decentralized
 * momentum updates of "DecentLaM: Decentralized Momentum SGD for Large-batch
 * Deep Training" (arXiv 2104.11981).
 *
 * One GPU simulates all n nodes.  The stacked arrays of the paper's appendix
 * "Preliminary" (x, m, gradient: n x d, row i = node i) live in device memory as
 * row-major fp32 with a row stride `ld >= d` (in elements).  A weight matrix W
 * (Sec. "Decentralized Momentum SGD", eq. (2)) is a neighbour list in CSR form
 * held in HOST memory: row i lists the j with w_ij > 0, i itself included.  A
 * time-varying W is `period` such lists stored phase after phase; iteration k
 * uses phase k mod period.
 *
 * Common rules
 *  - Every function returns DL_OK (0) or a negative dl_status; nothing aborts,
 *    prints or throws.  dl_last_error() gives a thread-local description of the
 *    last failure on the calling thread.
 *  - The caller owns every buffer.  The library allocates no device memory and keeps no state
 *    between calls, with one exception that no result depends on: kernel variants whose on-chip
 *    tile exceeds 48 KiB need a driver attribute raised once per device, and the library remembers
 *    per variant and device that it has done so (likewise how many workgroups of local_grad_lsq's
 *    widest sweep a device holds at once).  One setting is kept: local_grad_lsq_poll_limit.
 *  - Device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and the call returns without synchronising.  Host
 *    arrays (the topology) are consumed before the call returns.
 *  - Arithmetic: inputs are promoted to fp64 in registers, every statement of
 *    the algorithm is evaluated in fp64, and each output element is rounded to
 *    fp32 once when stored.
 */
#ifndef DECENTLAM_H
#define DECENTLAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DL_OK = 0,
    DL_EINVAL = -1, /* bad scalar/pointer argument                                  */
    DL_ETOPO = -2,  /* neighbour list malformed or beyond DL_MAX_NODES / DL_MAX_NNZ* */
    DL_ECAP = -3,   /* an output or workspace capacity is too small                 */
    DL_EHIP = -4,   /* a HIP runtime call failed (text in dl_last_error)            */
    DL_EALIAS = -5  /* x, m, g (or A, y, x, g) overlap                              */
} dl_status;

typedef enum {
    DL_TOPO_RING = 0,        /* N_i = {i, i-1, i+1}                    (appendix "Network topologies") */
    DL_TOPO_EXP_STATIC = 1,  /* N_i = {i} U {i + 2^t}, t = 0..tau-1    (exponential graph, directed)   */
    DL_TOPO_EXP_ONEPEER = 2, /* phase p: N_i = {i, i + 2^p}, period tau (one-peer exponential graph)   */
    DL_TOPO_EXP_SYM = 3,     /* N_i = {i} U {i + 2^t, i - 2^t}          (symmetric exponential graph)   */
    DL_TOPO_MESH = 4,        /* R x C grid, 4-neighbourhood, no wrap-around; R = largest divisor of n
                                not above sqrt(n), node i at (i / C, i % C)                             */
    DL_TOPO_BIPARTITE_MATCH = 5 /* per phase a seeded random perfect matching (topology_build_ex)      */
} dl_topo_kind;             /* tau = floor(log2(n-1)) + 1; all indices mod n */

/* Storage format of the gradient operand of the *_g16, *_multi and *_ex calls. */
typedef enum {
    DL_GRAD_F32 = 0,
    DL_GRAD_BF16 = 1,   /* upper 16 bits of the fp32 pattern */
    DL_GRAD_F16 = 2     /* IEEE binary16                      */
} dl_grad_format;

/* properties reported by topology_build (every phase has the property) */
#define DL_FLAG_ROW_STOCHASTIC 1u /* |sum_j w_ij - 1| <= 1e-6 for all i  (Assumption A.3: W 1 = 1) */
#define DL_FLAG_COL_STOCHASTIC 2u /* |sum_i w_ij - 1| <= 1e-6 for all j                            */
#define DL_FLAG_SYMMETRIC 4u      /* w_ij == w_ji                         (Assumption A.3)         */

/* limits of the step kernels: the phase's neighbour list travels in the kernel arguments */
#define DL_MAX_NODES 256
#define DL_MAX_NNZ 512            /* entries per phase, arbitrary weights                                 */
#define DL_MAX_NNZ_PALETTE 1536   /* entries per phase when it holds at most DL_MAX_WEIGHT_VALUES distinct */
#define DL_MAX_WEIGHT_VALUES 64   /* weight values (true of every topology topology_build produces)       */
#define DL_MAX_NNZ_ROW_WEIGHTS 2816 /* entries per phase when, besides, every row carries one value only   */
                                  /* (uniform 1/|N_i| rows: the exponential graph up to 256 nodes)        */

/*
 * topology_build -- neighbour lists and weights of the paper's topologies
 * (appendix "Network topologies"; one-peer graph: Introduction).
 *
 * Host-only, integer work.  Row order: self first, then ring: i-1, i+1;
 * exponential: ascending hop (symmetric: +2^t before -2^t); mesh: up, down, left, right;
 * match: the partner.  Duplicates (tiny n) are dropped keeping the first occurrence.
 * Weights: the undirected kinds follow the Metropolis-Hastings rule the paper cites,
 * w_ij = 1 / (1 + max(deg_i, deg_j)), w_ii = 1 - sum_j w_ij (deg counts neighbours other than
 * i); where all neighbours of i share its degree this is (float)1 / (float)|N_i| and is
 * evaluated as such.  The two directed exponential kinds carry the uniform 1 / |N_i|.
 *
 *   row_ptr  [out] period*(n+1) absolute offsets into col_idx / w, phase-major.
 *                  Pass NULL (with col_idx = w = NULL) to query sizes only.
 *   col_idx, w [out] nnz_out entries each.
 *   row_ptr_cap, nnz_cap  capacities in elements.
 *   period_out, nnz_out, flags_out [out] always written on DL_OK and DL_ECAP.
 * Errors: DL_EINVAL (n < 1, unknown kind, NULL out pointers), DL_ECAP.
 */
int topology_build(int kind, int32_t n,
                   int32_t* row_ptr, int64_t row_ptr_cap,
                   int32_t* col_idx, float* w, int64_t nnz_cap,
                   int32_t* period_out, int64_t* nnz_out, uint32_t* flags_out);

/*
 * topology_build_ex -- the same with the parameters of the randomised kind.
 * DL_TOPO_BIPARTITE_MATCH (appendix "Network topologies", last item): `phases` matchings,
 * iteration k uses matching k mod phases.  Matching p comes from a Fisher-Yates shuffle of
 * 0..n-1 driven by splitmix64 seeded with seed ^ (0xD1B54A32D192ED03 * (p + 1)) (from the
 * top index t = n-1 down to 1, swap with index next() % (t + 1)); shuffled position q is
 * paired with position q + n/2; with odd n the last position stays alone.  Every node derives
 * the same matching from the same seed, which is what the paper asks for.  Weights 1/2, 1/2.
 * Other kinds ignore seed and phases.  Additional error: DL_EINVAL if phases < 1 for the match.
 */
int topology_build_ex(int kind, int32_t n, uint64_t seed, int32_t phases,
                      int32_t* row_ptr, int64_t row_ptr_cap,
                      int32_t* col_idx, float* w, int64_t nnz_cap,
                      int32_t* period_out, int64_t* nnz_out, uint32_t* flags_out);

/*
 * topology_metropolis -- Metropolis-Hastings weights (the rule above) for a caller-supplied
 * undirected graph: one phase in CSR form, every row containing i itself, j in N_i iff i in N_j.
 *   w [out] one weight per entry of col_idx, in the caller's order.   flags_out may be NULL.
 * Errors: DL_EINVAL, DL_ETOPO (empty row, index out of range, duplicate, missing self, not undirected).
 */
int topology_metropolis(int32_t n, const int32_t* row_ptr, const int32_t* col_idx,
                        float* w, uint32_t* flags_out);

/*
 * decentlam_step -- one iteration of Algorithm 2 (DecentLaM) for all nodes:
 *     z_i  = sum_{j in N_i} w_ij (x_j - gamma g_j)          partial averaging, eq. (3)
 *     gt_i = (x_i - z_i) / gamma                             corrected gradient (equation after
 *                                                            the "Efficient implementation" paragraph)
 *     m_i <- beta m_i + gt_i ;  x_i <- x_i - gamma m_i       momentum and model update
 * fused into one pass that reads x, m, g once and writes x, m once (20 bytes
 * per node-element).
 *
 *   x, m   [in,out] device, n x d fp32, row stride ld; updated in place.
 *   g      [in]     device, same shape and stride; the stochastic gradients.
 *   row_ptr, col_idx, w, period  [in] host; W as described above.  Row sums must
 *                   be 1 within 1e-6; weights finite and > 0; no duplicate j in a row.
 *   gamma > 0 finite; 0 <= beta < 1; k >= 0 selects phase k mod period.
 *   The caller zeroes m before iteration 0 (Algorithm 2, initialisation).
 * d == 0 is a successful no-op.  Any alignment and any ld >= d are accepted
 * (unaligned heads/tails fall back to narrower loads); for full speed let rows start on
 * 128-byte boundaries (16-byte aligned bases, ld a multiple of 32), and for arrays of
 * 65536 columns or more on 64 KiB boundaries (64 KiB-aligned bases, ld a multiple of
 * 16384): the step then writes whole 64 KiB-aligned address pairs (A, A + 32 KiB), worth
 * about 10 % at every node count (measured at n = 32, d = 25.6 M: 2.51 instead of 2.80 ms).  Avoid an ld that
 * is a multiple of 127 or 129 times 16384: the rows of a column then fall on the same memory channels
 * (32 nodes x 1 M columns: 161 instead of 110 us with ld = 129 * 16384; 2 to 6 % at 25 M columns).  Rows that
 * alternate between such boundaries and their midpoints (ld an odd multiple of 8192, e.g. a contiguous
 * 32 x 25.6 M array; 17 to 32 nodes, x, m, g placed alike modulo 64 KiB) are served by a kernel of their
 * own that loads and stores half of each odd row's accesses one 64 KiB unit ahead / late: 2.64 ms there.
 * On 33 to 128 nodes the 64 KiB alignment also selects a kernel that uses an on-chip tile of half the width
 * twice per 256 columns: 6.3-6.5 instead of 5.9-6.2 TB/s up to 64 nodes (two workgroups per CU instead of
 * one; there rows on any 512-byte boundary select it, at 5.8-6.2 TB/s), 5.4-5.7 instead of 5.0-5.2 beyond
 * (16-byte instead of 8-byte accesses).
 * Dense graphs (23 <= n <= 32 with 46 - n or more entries per row on average: 14 at n = 32, all
 * 23 at n = 23; 33 <= n <= 48 with 38 - n / 4 or more; this holds for every step entry point): the partial averaging runs as an fp64 matrix product on the matrix cores
 * instead of neighbour by neighbour (all-to-all at n = 32, d = 25.6 M: 2.7 instead of 3.5 ms).
 * The sums are then taken in the instruction's order, not list order (differences in the last
 * bits of fp64, before the one rounding to fp32), and absent pairs enter with weight zero: a
 * non-finite value in one node's column turns that column non-finite for every node, neighbour
 * or not.
 * Errors: DL_EINVAL, DL_ETOPO, DL_EALIAS, DL_EHIP.
 */
int decentlam_step(float* x, float* m, const float* g,
                   int32_t n, int64_t d, int64_t ld,
                   const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                   float gamma, float beta, int64_t k, void* stream);

/*
 * dmsgd_step -- one iteration of Algorithm 1 (DmSGD), same arguments:
 *     m_i <- beta m_i + g_i ;  h_i = x_i - gamma m_i ;  x_i <- sum_{j in N_i} w_ij h_j
 */
int dmsgd_step(float* x, float* m, const float* g,
               int32_t n, int64_t d, int64_t ld,
               const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
               float gamma, float beta, int64_t k, void* stream);

/*
 * topology_pack, *_step_packed -- W validated and encoded once instead of at every call.
 *
 * The step calls above take W as three flat host arrays (the fields a `dl_topology { n, period, row_ptr,
 * col_idx, w }` struct would carry, passed one by one) and check and encode the phase in use on every call:
 * O(entries) host work per iteration, which shows where a step is only microseconds long.  topology_pack
 * does that work for all `period` phases once and writes the result into a caller-owned host buffer of
 * topology_pack_bytes(n, period) bytes (4-byte aligned; an opaque blob that holds no pointers: it may be
 * copied, must not be edited, and is only valid for the library build that wrote it).  The *_step_packed
 * calls take that buffer in place of (row_ptr, col_idx, w, period); iteration k uses phase k mod period as
 * before.  Results are bit-identical to the flat calls.  The library keeps no reference to the buffer and
 * no other state: the buffer is consumed before the call returns.
 * Errors: topology_pack as the W checks of decentlam_step (DL_EINVAL, DL_ETOPO), DL_ECAP if the buffer is
 *         too small; *_step_packed as their flat forms, DL_ETOPO if the buffer was not written by
 *         topology_pack or describes another node count.  topology_pack_bytes returns 0 for n < 1,
 *         n > DL_MAX_NODES or period < 1.
 */
size_t topology_pack_bytes(int32_t n, int32_t period);
int topology_pack(int32_t n, const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  void* packed, size_t packed_bytes);
int decentlam_step_packed(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                          const void* packed, float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_packed(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                      const void* packed, float gamma, float beta, int64_t k, void* stream);
int dsgd_step_packed(float* x, const float* g, int32_t n, int64_t d, int64_t ld,
                     const void* packed, float gamma, int64_t k, void* stream);

/*
 * topology_pack_device, *_step_dev -- graphs beyond the limits above: up to DL_MAX_NODES_DEVICE nodes,
 * neighbour lists of any length with arbitrary weights (eq. (2) asks nothing more of W than its sparsity
 * pattern and weights).  The lists live in DEVICE memory: topology_pack_device validates all phases on the host
 * (the W rules of decentlam_step) and copies them, encoded, into a caller-owned device buffer of
 * topology_device_bytes(n, period, total entries over all phases) bytes, 8-byte aligned.  It is a set-up call:
 * the copy is synchronous (do not call it under graph capture).  It fills a small host descriptor that the
 * *_step_dev calls take; the descriptor holds the device pointer and must not outlive the buffer.
 * The step is the same in-place, single-pass, fp64-in-registers update (20 bytes per node-element), on a kernel
 * built for reach rather than speed: its tile narrows as n grows (64 columns up to 256 nodes, 32 up to 512, 16
 * up to 1024), so rows are touched 256, 128 or 64 bytes at a time.  Graphs that fit the ordinary calls should
 * use them.  fp32 gradients, row-major arrays; decentlam, dmsgd and dsgd.
 * Errors: DL_EINVAL, DL_ETOPO (also: n > DL_MAX_NODES_DEVICE, descriptor not written by topology_pack_device or
 *         for another node count), DL_ECAP (device buffer too small), DL_EALIAS, DL_EHIP.
 */
#define DL_MAX_NODES_DEVICE 1024
typedef struct {
    uint32_t magic;          /* set by topology_pack_device */
    int32_t n, period;
    int32_t reserved;
    const void* device;      /* the caller's device buffer */
    uint64_t device_bytes;   /* bytes of it in use */
} dl_device_topology;
size_t topology_device_bytes(int32_t n, int32_t period, int64_t nnz_total);
int topology_pack_device(int32_t n, const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                         void* device_buffer, size_t device_bytes, dl_device_topology* out);
int decentlam_step_dev(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                       const dl_device_topology* W, float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_dev(float* x, float* m, const float* g, int32_t n, int64_t d, int64_t ld,
                   const dl_device_topology* W, float gamma, float beta, int64_t k, void* stream);
int dsgd_step_dev(float* x, const float* g, int32_t n, int64_t d, int64_t ld,
                  const dl_device_topology* W, float gamma, int64_t k, void* stream);

/*
 * decentlam_step_xprev -- DecentLaM in its momentum-free form (appendix "Reformulation of
 * DecentLaM"): with m^k = (x^{k-1} - x^k) / gamma_{k-1} eliminated,
 *     x^{k+1} = W (x^k - gamma_k g^k) + beta (gamma_k / gamma_{k-1}) (x^k - x^{k-1}).
 * The state is the pair (x^k, x^{k-1}) instead of (x^k, m^k); m^0 = 0 corresponds to
 * x^{-1} = x^0.  Same iterates as decentlam_step in exact arithmetic.
 *
 *   x      [in]     device, n x d fp32 (ld): x^k, not modified.
 *   x_prev [in,out] device, same shape: x^{k-1} on entry, x^{k+1} on exit.  The caller swaps the
 *                   roles of the two buffers after every call.
 *   gamma_prev      the learning rate of the previous call (pass gamma for a constant rate).
 * Reads x, x_prev, g and writes one array: 16 bytes per node-element.  Other arguments,
 * conventions and errors as decentlam_step.
 */
int decentlam_step_xprev(const float* x, float* x_prev, const float* g,
                         int32_t n, int64_t d, int64_t ld,
                         const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                         float gamma, float gamma_prev, float beta, int64_t k, void* stream);

/*
 * decentlam_step_blocked, dmsgd_step_blocked -- the same iterations on arrays held in a blocked
 * layout: the columns are cut into blocks of `bw`; a block is a row-major n x bw matrix (row stride
 * bw) and the blocks follow one another, so element (i, c) of x lives at
 *     x[((c / bw) * n + i) * bw + c % bw]
 * (the last block may hold fewer than bw columns; its rows still start bw apart).  Each array is
 * ceil(d / bw) * n * bw elements at most.  Nothing else changes: same arithmetic, same 20 bytes per
 * node-element.  The layout keeps the n rows a workgroup works on within n * bw * 4 bytes instead of
 * n rows that are d * 4 bytes apart; with row starts 32 KiB apart (bw = 8192) a tile's writes fill
 * whole 64 KiB-aligned address pairs whatever d is.  Up to 32 nodes it runs at the rate of the
 * row-major call with 64 KiB-aligned rows (measured at n = 32: 6.5 TB/s both) and 10 % faster than a
 * row-major call whose rows are not so aligned; at 64 nodes and more it is the faster layout
 * (n = 128: 6.4 instead of 5.5 TB/s).  Let bw be a multiple of 64 and the bases 16-byte aligned for
 * full-width accesses.  Errors as decentlam_step; bw < 1 is DL_EINVAL.
 */
int decentlam_step_blocked(float* x, float* m, const float* g,
                           int32_t n, int64_t d, int64_t bw,
                           const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                           float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_blocked(float* x, float* m, const float* g,
                       int32_t n, int64_t d, int64_t bw,
                       const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                       float gamma, float beta, int64_t k, void* stream);

/*
 * decentlam_step_ex, dmsgd_step_ex, decentlam_step_xprev_ex -- the general forms: any combination of
 * layout (row-major or blocked) and gradient format.  The simpler calls above are special cases.
 *
 *   layout->bw == 0   row-major arrays: x, m with row stride layout->ld, g with row stride
 *                     layout->ldg (elements of its format; < 0 means "same as ld").
 *   layout->bw  > 0   blocked layout with blocks of bw columns for all three arrays (ld, ldg ignored).
 *   layout->g_format  a dl_grad_format; g points to elements of that format.
 * decentlam_step_xprev_ex with 16-bit gradients in the blocked layout is the leanest iteration the
 * library offers: 14 bytes per node-element (read x^k, x^{k-1} fp32 and g 16-bit, write x^{k+1}).
 * Errors as the special cases; a NULL layout or bw < 0 is DL_EINVAL.
 */
typedef struct {
    int32_t g_format;
    int64_t ld;
    int64_t ldg;
    int64_t bw;
} dl_layout;
int decentlam_step_ex(float* x, float* m, const void* g,
                      int32_t n, int64_t d, const dl_layout* layout,
                      const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                      float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_ex(float* x, float* m, const void* g,
                  int32_t n, int64_t d, const dl_layout* layout,
                  const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  float gamma, float beta, int64_t k, void* stream);
int decentlam_step_xprev_ex(const float* x, float* x_prev, const void* g,
                            int32_t n, int64_t d, const dl_layout* layout,
                            const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                            float gamma, float gamma_prev, float beta, int64_t k, void* stream);

/*
 * decentlam_step_multi_ex, dmsgd_step_multi_ex -- the multi-tensor calls in their general form: tensor
 * table and per-tensor sums as decentlam_step_multi, layout and gradient format from a dl_layout.
 * In the blocked layout (layout->bw > 0) the table starts at column 0 (offsets[0] == 0), and with
 * norms != NULL the block width must be a multiple of 256 and x, m 16-byte aligned (g: 4 elements),
 * so that whole tiles line up with the columns (DL_EINVAL otherwise).
 */
int decentlam_step_multi_ex(float* x, float* m, const void* g,
                            int32_t n, const dl_layout* layout,
                            int32_t num_tensors, const int64_t* offsets,
                            double* norms, void* workspace, size_t workspace_bytes,
                            const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                            float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_multi_ex(float* x, float* m, const void* g,
                        int32_t n, const dl_layout* layout,
                        int32_t num_tensors, const int64_t* offsets,
                        double* norms, void* workspace, size_t workspace_bytes,
                        const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                        float gamma, float beta, int64_t k, void* stream);

/*
 * awc_dmsgd_step, da_dmsgd_step -- two sibling methods of the paper's comparison that reuse the
 * same fused gather-mix pass (Sec. "Experiments", list of compared algorithms).  The paper
 * describes them in a sentence each and prints no recursion; the library implements this reading:
 *   AWC-DmSGD  (momentum on the adaptation-with-combination form x <- W x - gamma grad, the
 *              recursion printed after the DSGD-as-SGD proposition):
 *                  m_i <- beta m_i + g_i ;  x_i <- sum_{j in N_i} w_ij x_j - gamma m_i
 *   DA-DmSGD   (Algorithm 1 with an additional partial average over the momentum):
 *                  mh_i = beta m_i + g_i ;  x_i <- sum_j w_ij (x_j - gamma mh_j) ;  m_i <- sum_j w_ij mh_j
 * Arguments, conventions and errors as dmsgd_step; 20 bytes per node-element (da_dmsgd_step uses
 * its on-chip tile twice, for x - gamma mh and then for mh).
 */
int awc_dmsgd_step(float* x, float* m, const float* g,
                   int32_t n, int64_t d, int64_t ld,
                   const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                   float gamma, float beta, int64_t k, void* stream);
int da_dmsgd_step(float* x, float* m, const float* g,
                  int32_t n, int64_t d, int64_t ld,
                  const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                  float gamma, float beta, int64_t k, void* stream);

/*
 * awc_dmsgd_step_ex, da_dmsgd_step_ex, awc_dmsgd_step_multi_ex, da_dmsgd_step_multi_ex -- the two sibling
 * methods in the general forms: layout (row-major or blocked) and gradient format (fp32, bf16, fp16) from a
 * dl_layout as decentlam_step_ex, tensor table and per-tensor sums of squares of g, the new m and the new x as
 * decentlam_step_multi_ex (for da_dmsgd the new m is the averaged one).  Arguments, conventions and errors as
 * those calls.
 */
int awc_dmsgd_step_ex(float* x, float* m, const void* g,
                      int32_t n, int64_t d, const dl_layout* layout,
                      const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                      float gamma, float beta, int64_t k, void* stream);
int da_dmsgd_step_ex(float* x, float* m, const void* g,
                     int32_t n, int64_t d, const dl_layout* layout,
                     const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                     float gamma, float beta, int64_t k, void* stream);
int awc_dmsgd_step_multi_ex(float* x, float* m, const void* g,
                            int32_t n, const dl_layout* layout,
                            int32_t num_tensors, const int64_t* offsets,
                            double* norms, void* workspace, size_t workspace_bytes,
                            const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                            float gamma, float beta, int64_t k, void* stream);
int da_dmsgd_step_multi_ex(float* x, float* m, const void* g,
                           int32_t n, const dl_layout* layout,
                           int32_t num_tensors, const int64_t* offsets,
                           double* norms, void* workspace, size_t workspace_bytes,
                           const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                           float gamma, float beta, int64_t k, void* stream);

/*
 * decentlam_step_g16, dmsgd_step_g16 -- Algorithm 2 / Algorithm 1 with the gradients held in a
 * 16-bit format, as they come out of a mixed-precision backward pass (the paper trains in mixed
 * precision, Sec. "Experiments", implementation details); x and m stay fp32.  Each g value is
 * widened exactly to fp32 on load, so the call computes what decentlam_step / dmsgd_step compute on
 * the widened array: 18 bytes per node-element instead of 20.
 *
 *   g         [in] device, n x d elements of `g_format` (a dl_grad_format), row stride ldg elements,
 *                  aligned to its element size.  DL_GRAD_F32 is accepted too (g with its own stride).
 *   ldg >= d.  For 8-byte accesses to g let rows of g start on 8-byte boundaries (ldg % 4 == 0).
 * Everything else as decentlam_step.
 */
int decentlam_step_g16(float* x, float* m, const void* g, int32_t g_format,
                       int32_t n, int64_t d, int64_t ld, int64_t ldg,
                       const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                       float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_g16(float* x, float* m, const void* g, int32_t g_format,
                   int32_t n, int64_t d, int64_t ld, int64_t ldg,
                   const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                   float gamma, float beta, int64_t k, void* stream);

/*
 * decentlam_step_multi, dmsgd_step_multi -- one iteration over a table of tensors (the layers of a
 * model, flattened and packed along the columns), optionally with per-tensor, per-node sums of
 * squares taken from the registers of the same pass.  Such layer-wise norms are what layer-wise
 * adaptive rate scaling, the companion of large-batch momentum SGD in the paper's comparison
 * (Sec. "Experiments"), consumes.  The update itself is the one of decentlam_step / dmsgd_step
 * applied to the columns [offsets[0], offsets[num_tensors]).
 *
 *   x, m      [in,out] device, n x ld fp32 arrays; column c of the table is x[i * ld + c].
 *   g         [in]     device, gradient in `g_format`, row stride ldg, same column numbering.
 *   offsets   [in]     host, num_tensors + 1 non-decreasing column offsets, 0 <= offsets[0],
 *                      offsets[num_tensors] <= min(ld, ldg); tensor t is [offsets[t], offsets[t+1])
 *                      (empty tensors allowed; sizes need not be multiples of anything).
 *   norms     [out]    device, num_tensors x n x 3 doubles, or NULL for none:
 *                      norms[(t*n + i)*3 + 0] = sum of g_i^2 over tensor t (the values as loaded),
 *                      ... + 1 = sum of the new m_i^2, ... + 2 = sum of the new x_i^2 (the stored
 *                      fp32 values, squared and added in fp64).  Deterministic: same inputs, same bits
 *                      (from 2^20 columns on: for arrays at the same addresses modulo 64 KiB, which
 *                      decide where the tiles of the launch begin and with them the order of the sums).
 *   workspace [scratch] device, 8-byte aligned, at least
 *                      decentlam_step_multi_workspace(n, offsets[num_tensors] - offsets[0], num_tensors)
 *                      bytes; needed only when norms != NULL (per-tile partial sums).
 * With norms == NULL this is a single fused launch like the flat call; with norms the step launch
 * also writes one small record per tile and a final per-tensor pass follows (one launch per 440
 * tensors; the table travels as kernel arguments: no host-to-device copy, capturable).
 * Errors: as decentlam_step; DL_ECAP if the workspace is too small; DL_EINVAL for a bad table.
 */
size_t decentlam_step_multi_workspace(int32_t n, int64_t d, int32_t num_tensors);
int decentlam_step_multi(float* x, float* m, const void* g, int32_t g_format,
                         int32_t n, int64_t ld, int64_t ldg,
                         int32_t num_tensors, const int64_t* offsets,
                         double* norms, void* workspace, size_t workspace_bytes,
                         const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                         float gamma, float beta, int64_t k, void* stream);
int dmsgd_step_multi(float* x, float* m, const void* g, int32_t g_format,
                     int32_t n, int64_t ld, int64_t ldg,
                     int32_t num_tensors, const int64_t* offsets,
                     double* norms, void* workspace, size_t workspace_bytes,
                     const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
                     float gamma, float beta, int64_t k, void* stream);

/*
 * dsgd_step -- one iteration of DSGD (eqs. (4)-(5), compact form x <- W (x - gamma g)), the
 * momentum-free method both algorithms reduce to at beta = 0 and the baseline of the paper's
 * linear-regression study.  Same conventions; there is no momentum array.  12 bytes per node-element.
 */
int dsgd_step(float* x, const float* g,
              int32_t n, int64_t d, int64_t ld,
              const int32_t* row_ptr, const int32_t* col_idx, const float* w, int32_t period,
              float gamma, int64_t k, void* stream);

/*
 * local_grad_lsq -- per-node least-squares gradient (appendix "Experimental
 * setting for linear regression"): for f_i(x) = (scale/2) ||A_i x - y_i||^2,
 *     res_i = A_i x_i - y_i ;  g_i = scale * A_i^T res_i ;  loss_i = (scale/2) ||res_i||^2
 *
 *   A  [in] device, n x b x d fp32: element (i, r, c) at A[(i*b + r)*ldA + c], ldA >= d.
 *   y  [in] device, n x b fp32, contiguous.
 *   x  [in] device, n x d fp32, row stride ld.     g [out] device, n x d fp32, row stride ld.
 *   loss [out] device, n fp32, or NULL.
 *   workspace [scratch] device, at least local_grad_lsq_workspace(n, b, d) bytes, 16-byte aligned;
 *             contents are undefined before and after the call (no initialisation is needed).
 * Deterministic: partial sums are combined in a fixed order.
 * The contraction is a batch of n matrix-vector products with no shared operand (every node has its own
 * A_i and x_i): 1 flop per byte of A at best, so the bound is HBM bandwidth and the kernels are built
 * around one streaming pass over A.  That pass is fastest with the rows of A on 16-byte boundaries (ldA a multiple
 * of 4, A 16-byte aligned; x and g may lie anywhere) and d <= 32768 (64 nodes of 4096 x 4096: 0.62 ms, 0.86 of the
 * HBM peak; 4096 x 4095 with ldA = 4096: 0.63 ms).  Rows of A on 8-byte boundaries only (8 nodes of 4096 x 7850,
 * contiguous: 0.19 ms, 0.67) or on none (4096 x 4095 with ldA = 4095: 1.05 ms, 0.51) are still read once, with
 * narrower accesses, up to d = 16384, so pad ldA where that is possible.  Rows of up to 1024 columns are handled a
 * wave per row (64 nodes of 32768 x 128: 0.78 of the peak, of 4096 x 1024: 0.85), at any alignment.  Between the
 * sizes named here the rate moves between 0.7 and 0.85 with how well d fills the kernel's shape (steps of 256
 * columns up to 2560, of 1024 up to 8192, of 4096 beyond; lowest, 0.56-0.6, just above 8192; rows off the 16-byte
 * boundaries: 0.8 up to 2048 columns, 0.65-0.75 up to 8192, 0.5-0.65 up to 16384).  Rows of 32772 to 262144 columns
 * (d a multiple of 4, rows of A on 16-byte boundaries) are still read once: the columns of a block of rows are split
 * over waves of several workgroups, which hand one another their shares of each row's dot product through the workspace
 * (8 nodes of 1024 x 65536: 0.35 ms, 0.76 of the peak; other shapes 0.6-0.78, beyond 131072 columns 0.6-0.67).
 * Those workgroups wait for one another, so a launch is sized to what the chip holds at once and every wait is
 * bounded: should the GPU be kept busy by other work for seconds on end, so that they cannot all run together, the
 * call gives up and leaves NaN in g and loss (of the nodes of the launch concerned and of those after it) instead
 * of hanging.  Wider rows than these limits take two passes over A at 0.3-0.35 of the peak.  No access
 * reaches past column d of a row in any case.
 * Products and sums run as fp64 fused multiply-adds on the vector units; the matrix cores are
 * not used: an MFMA tile would have one useful column in sixteen, and for fp32 / fp64 the matrix and
 * vector peaks of this chip are equal.
 * Errors: DL_EINVAL (NULL, n < 1, b < 1, d < 0, ldA < d, ld < d, scale not finite),
 *         DL_ECAP (workspace too small), DL_EALIAS (g overlaps an input), DL_EHIP.
 */
size_t local_grad_lsq_workspace(int32_t n, int32_t b, int64_t d);
int local_grad_lsq(const float* A, const float* y, const float* x,
                   float* g, float* loss,
                   int32_t n, int32_t b, int64_t d, int64_t ldA, int64_t ld,
                   float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * local_grad_lsq_poll_limit -- how long the waves of local_grad_lsq's sweep over rows of more than 32768 columns
 * wait for one another (see local_grad_lsq): the number of polls after which a wave gives up, process-wide, the one
 * setting the library keeps between calls.  The default, 2097152, is seconds.  polls < 0 restores the default;
 * 0 makes every wave that finds a share missing give up at once, which is how the tests reach the path that
 * answers with NaN instead of numbers (every kernel still runs to its end).  Returns the previous value.
 */
int local_grad_lsq_poll_limit(int polls);

/*
 * local_grad_lsq_static -- local_grad_lsq for callers that cannot allocate or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * results bit for bit; the partial sums live in an array of DL_STATIC_SCRATCH_BYTES that is part of
 * the library's device image (every GPU the library runs on holds its own copy until the process
 * ends).  The call allocates nothing and frees nothing.
 *   Limit: the partial sums of the kernels this shape and alignment select must fit
 *   DL_STATIC_SCRATCH_BYTES (32 MiB).  With one sweep over A (see local_grad_lsq)
 *   that is about n * max(1, 512 / n) * (d + 1) * 8 bytes (n = 64 nodes of 4096 x 4096: 16.8 MB; up to d = 256,
 *   where 2048 takes the place of 512, at most 4.2 MB), never
 *   more than local_grad_lsq_workspace(n, b, d).  Larger problems return DL_ECAP (nothing is launched)
 *   and belong to local_grad_lsq.
 *   All calls on one GPU share that GPU's array: calls that may overlap in time (different streams,
 *   different threads) race on it and must be serialised by the caller.  The array keeps the last
 *   call's contents; every call writes each partial sum before it reads it (and, for rows of more than 32768
 *   columns, marks the waves' exchange slots empty with a fill kernel of its own first), so nothing needs clearing.
 *   The first call on a device looks the array's address up (this may load the library's device
 *   code): make it once outside of graph capture.
 * Arguments and the other errors as local_grad_lsq.
 */
#define DL_STATIC_SCRATCH_BYTES (32u << 20)
int local_grad_lsq_static(const float* A, const float* y, const float* x,
                          float* g, float* loss,
                          int32_t n, int32_t b, int64_t d, int64_t ldA, int64_t ld,
                          float scale, void* stream);

/*
 * local_grad_lsq_rows -- the stochastic (mini-batch) version: node i's sample xi_i (Algorithms 1
 * and 2, "Sample xi_i") is a list of bs row indices into its local data, drawn by the caller:
 *     g_i = scale * sum_{t < bs} a_t (a_t . x_i - y_i[r_t]),  r_t = rows[i*bs + t],  a_t = A_i[r_t, :]
 *     loss_i = (scale/2) * sum_t (a_t . x_i - y_i[r_t])^2
 * Repeated indices are allowed (sampling with replacement) and count as often as they appear.
 *   rows [in] device, n x bs int32 with values in [0, b); values outside are clamped into the range.
 *   workspace: at least local_grad_lsq_workspace(n, bs, d) bytes.
 * Everything else as local_grad_lsq.  Additional errors: DL_EINVAL (rows NULL, bs < 1).
 */
int local_grad_lsq_rows(const float* A, const float* y, const float* x,
                        float* g, float* loss,
                        int32_t n, int32_t b, int64_t d, int64_t ldA, int64_t ld,
                        const int32_t* rows, int32_t bs,
                        float scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * decentlam_stats -- diagnostics of the stacked state, one pass over x (and m):
 *     out[0] = sum_i ||x_i - xbar||^2,  xbar = (1/n) sum_i x_i   (consensus distance; xbar as in
 *                                                                 the appendix "Preliminary")
 *     out[1] = ||xbar||^2
 *     out[2] = sum_i ||x_i - ref||^2,  out[3] = ||ref||^2         (0 if ref == NULL); the relative
 *              error of the appendix "Experimental setting for linear regression",
 *              (1/n) sum_i ||x_i - x*||^2 / ||x*||^2, is out[2] / (n * out[3]) with ref = x*
 *     out[4] = ||m||_F^2                                          (0 if m == NULL)
 *
 *   x [in] device n x d fp32 (row stride ld); m [in] same shape or NULL; ref [in] device, d fp32, or NULL.
 *   out [out] device, 5 doubles.  workspace [scratch] device, decentlam_stats_workspace(n, d) bytes.
 * fp64 sums combined in a fixed order (bit-reproducible).  d == 0 yields zeros.
 * Errors: DL_EINVAL, DL_ECAP, DL_EHIP.
 */
size_t decentlam_stats_workspace(int32_t n, int64_t d);
int decentlam_stats(const float* x, const float* m, const float* ref,
                    int32_t n, int64_t d, int64_t ld,
                    double* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dl_calibration_stream -- no part of the method: a bare stream with the step kernel's access pattern,
 * which benchmarks use as the achievable-bandwidth denominator beside the published HBM peak.  One
 * workgroup per 256 columns of all n rows, the loads of x, g, m up front, one barrier, the stores of m and
 * x; no on-chip tile, no neighbour list.
 *   kind  0: x <- x + g / 2, m <- m / 2 + g (3 reads + 2 writes, 20 bytes per node-element);
 *         1: the three reads only (12 bytes); 2: the two writes only (8 bytes; x and m are overwritten).
 *   split 0: tile t owns columns [256 t, 256 t + 256); 1: the column order of the step's large launches
 *         (two 512-byte segments 32 KiB apart inside 64 KiB units of 16384 columns).
 *   x, m, g  device, n x d fp32 with row stride ld, n <= 32, 16-byte aligned, ld a multiple of 4.
 *   columns_out [out, host] columns actually covered: whole tiles only (d rounded down to a multiple of 256,
 *         or of 16384 in the split order); the rest is left untouched.
 * Errors: DL_EINVAL, DL_EHIP.
 */
int dl_calibration_stream(int kind, int split, float* x, float* m, const float* g,
                          int32_t n, int64_t d, int64_t ld, int64_t* columns_out, void* stream);

/* Description of the last failure on the calling thread ("" if none). Never NULL. */
const char* dl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DECENTLAM_H */
