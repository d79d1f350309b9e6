/*
 * solon.h - C ABI of the MI355X (gfx950) implementation of Solon's linear block code:
 * redundant-gradient encode at the compute nodes and locate + decode at the parameter server.
 *
 * Notation is the paper's (Sec. 3.1-3.4): P compute nodes, B per-batch gradients g_1..g_B of
 * dimension d, at most s Byzantine nodes, compression ratio m (the paper's r_c), message length
 * d_c = ceil(d / m), redundancy r = 2 s + m (Thm. 2), q groups ("blocks") of nodes that hold the
 * same gradients, evaluation points w_1..w_P, projection vector f, honest messages Z, received
 * matrix R = Z + N, located set V, decoded sum u = G 1_P.
 *
 * Layout.  Every matrix is row-major with one ROW per node or per batch (the paper writes nodes as
 * columns): G is B x d, Z and R are P x d_c, contiguous along the coordinate axis, row strides given
 * in elements.  Coordinate c of a gradient belongs to chunk p = c / m, coefficient l = c % m.
 *
 * Pointers.  "device" = memory of the current HIP device, "host" = ordinary host memory.  The caller
 * owns every buffer it passes.  The library owns only the plan and the plan's small device workspace
 * (projection partial sums, located set, recombination table), allocated once by
 * solon_plan_create and released by solon_plan_destroy; no call allocates per invocation.
 *
 * Streams.  hip_stream is a hipStream_t passed as void* (NULL = the default stream).  All kernels
 * of a call are enqueued on it in order; a call returns without waiting unless it has to hand a
 * result back through a host pointer.  One locate -> decode pair may be in flight per plan.
 * The calls that take no host output (solon_encode; solon_locate, solon_locate_decode and
 * solon_decode_majority with NULL host pointers; solon_decode with n_byz < 0) allocate nothing,
 * issue no memsets and never wait for the host: they can be recorded into a HIP graph and replayed
 * (run each once eagerly first, so that the one-time occupancy queries are not part of the capture).
 *
 * Alignment.  Any element-aligned pointers and strides are accepted.  The fastest kernels need 16-byte
 * aligned rows: G, Z / R, f and u aligned to 16 bytes and row strides that are multiples of 16 bytes
 * (ldg a multiple of 4 fp32 or 8 bf16 elements, ldz / ldr a multiple of 4).  Other layouts (an odd d with
 * unpadded rows, say) run element-wise kernels at about three quarters of that speed; padding the row
 * strides is the cheap cure.
 *
 * Errors.  Every function returns SOLON_OK or a negative solon_status; nothing throws or aborts.
 * On error the outputs are unspecified, but no access outside the given extents is made.
 * solon_last_error() gives a thread-local description of the last failure.
 */
#ifndef SOLON_H
#define SOLON_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct solon_plan solon_plan; /* opaque; immutable after creation except for its workspace */

enum solon_status {
  SOLON_OK = 0,
  SOLON_E_INVAL = -1,   /* null pointer, P < 1, d < 1, m < 1, s < 0, bad dtype, bad group table, bad stride,
                           a group larger than SOLON_MAX_GROUP, 2 s + m >= SOLON_MAX_GROUP, m > 16                                             */
  SOLON_E_BOUND = -2,   /* a group has fewer than 2 s + m nodes (Thm. 2) or s > (P - m) / 2 (its corollary) */
  SOLON_E_POINTS = -3,  /* an evaluation point is zero, non-finite, or repeated within a group (Sec. 3.4)  */
  SOLON_E_DECODE = -4,  /* some group cannot be explained by <= s corrupted nodes                          */
  SOLON_E_NUMERIC = -5, /* the m x m Vandermonde chosen for psi is too ill-conditioned to invert in fp32    */
  SOLON_E_HIP = -6      /* a HIP runtime call failed, or no device workspace exists (no GPU)                */
};

enum solon_dtype { SOLON_F32 = 0, SOLON_BF16 = 1 }; /* element type of G; Z, R, f, u are always fp32 */

enum solon_query {
  SOLON_Q_GROUPS = 0,      /* q                                                   */
  SOLON_Q_REDUNDANCY = 1,  /* r = 2 s + m                                         */
  SOLON_Q_MESSAGE_LEN = 2, /* d_c = ceil(d / m)                                   */
  SOLON_Q_MAX_GROUP = 3,   /* largest group size                                  */
  SOLON_Q_WORKSPACE = 4,   /* bytes of device workspace owned by the plan         */
  SOLON_Q_HAS_DEVICE = 5,  /* 1 if the device workspace was allocated, else 0     */
  SOLON_Q_LAST_REDO = 6,   /* 1 if the last solon_locate_decode on this plan had to repeat the recombination because one of
                              the guessed rows was located (waits for the device; a diagnostic, not part of the path)     */
  SOLON_Q_LIMIT_GROUP = 7, /* largest group the library handles (SOLON_MAX_GROUP); plan may be NULL                        */
  SOLON_Q_LIMIT_M = 8,     /* largest compression ratio m with compiled kernels; plan may be NULL                          */
  SOLON_Q_LAST_ONE_PASS = 9 /* 1 if the last solon_locate_decode on this plan ran the one-pass kernel, 0 if it took the two passes */
};

#define SOLON_MAX_GROUP 64 /* nodes per group handled by the single-wavefront locator */

/*
 * Allocation A and encoder weights (Sec. 3.4, "Linear Block Code": A = I_q (x) 1_{r x r},
 * W_j = I_{d_c} (x) [1, w_j, ..., w_j^{m-1}]).  Checks Thm. 2 (every group has >= 2 s + m nodes)
 * and its corollary (s <= (P - m) / 2).
 *   group_of_node  host int32[P], group index of each node, or -1 for a node that takes no part;
 *                  NULL = the default: q = floor(P / r) consecutive blocks, sizes differing by at
 *                  most one, larger blocks first (exactly the paper's blocks when r divides P).
 *   group_of_batch host int32[B], group whose nodes all compute gradient k; NULL = same as
 *                  group_of_node (requires B == P and no idle node).
 *   w              host float[P] evaluation points; NULL = Chebyshev-type points in (-1, 1),
 *                  one set per group size (see solon_default_points).
 * All three arrays are copied.  Creation succeeds without a GPU (host queries then work, compute
 * calls return SOLON_E_HIP).
 */
int solon_plan_create(solon_plan** out, int P, int B, int s, int m, int64_t d, int grad_dtype,
                      const int32_t* group_of_node, const int32_t* group_of_batch, const float* w);
void solon_plan_destroy(solon_plan* plan);
int solon_plan_query(const solon_plan* plan, int what, int64_t* value);
/* Copies of the plan's tables into host arrays: node -> group (int32[P]) and evaluation points (float[P]). */
int solon_plan_groups(const solon_plan* plan, int32_t* group_of_node);
int solon_plan_points(const solon_plan* plan, float* w);

/* Default evaluation points for a group of r_g nodes (host only, no GPU needed): the K = 2 ceil(r_g / 2)
 * Chebyshev nodes cos((2 i - 1) pi / (2 K)), i = 1..K, computed in double and rounded to float; for odd r_g
 * the node with 0-based index K / 2 is left out.  out: host float[r_g]. */
int solon_default_points(int r_g, float* out);

/*
 * E: the messages of all P nodes (Sec. 3.4: z_j = W_j Y_j 1_P; the group sum Y_j 1_P is formed once per
 * group and never stored).  Reads each element of G once, writes each element of Z once.
 *   G   device, B rows x d elements of the plan's grad dtype, row stride ldg elements (ldg >= d)
 *   Z   device, P rows x d_c fp32, row stride ldz elements (ldz >= d_c); rows of idle nodes are not written
 * Coordinates c >= d of the last chunk count as zero.  Group sums and the Horner evaluation are fp32.
 * Large inputs run on a persistent grid whose blocks align their read and write phases through counters in the
 * plan's workspace (so do solon_decode, solon_locate_decode and solon_decode_majority): overlapping two such calls on
 * different streams - of one plan or of two, since each of these grids is sized to fill the chip - stays correct (every wait
 * is bounded, and after the first wait that runs into the bound a launch stops waiting altogether) but loses that
 * alignment, i.e. runs like the flat kernels.
 */
int solon_encode(const solon_plan* plan, const void* G, int64_t ldg, float* Z, int64_t ldz, void* hip_stream);

/*
 * The projection vector of phi, drawn on the device (Sec. 3.4: f is generated inside phi, i.i.d. normal with mean one and
 * unit variance): f[p] = 1 + z_p with z_p standard normal, a pure function of (seed, p) - Philox-4x32-10 on the counter
 * (p / 4, 0, 0, 0) under the key (low, high word of seed), Box-Muller on the two word pairs in double precision, rounded to
 * float once - so that a fresh f costs one call and no host traffic, and any implementation of the same recipe reproduces
 * it.  Draw it AFTER R has arrived: a sender that knows f can hide a corruption from the projection.
 *   f   device, d_c fp32 (written)
 */
int solon_draw_projection(uint64_t seed, int64_t d_c, float* f, void* hip_stream);

/*
 * phi for all q groups (Sec. 3.4; Lemma 1): projections rho_j = sum_p f_p R[j][p] accumulated in fp64 with
 * a fixed reduction order, then per group the error-locator system
 *   [W_{m+s-1}, -W_{s-1} .* (rho 1^T)] a = rho .* w^s
 * solved in fp64 by one wavefront; nodes whose projection departs from the recovered degree-(m-1)
 * polynomial by more than 1e-4 x (median |rho| of the group) form V.  A non-finite projection is located at once.
 *   R        device, P x d_c fp32, row stride ldr
 *   f        device, d_c fp32, drawn by the caller i.i.d. N(1, 1)
 *   byz_idx  host int32[>= q * s] or NULL: receives V as ascending global node indices
 *   n_byz    host int32* or NULL: receives |V|
 *   rho_out  host double[P] or NULL: receives the projections
 * V, the honest rows chosen for psi and psi's coefficient table stay in the plan's device workspace for
 * solon_decode.  If any host output pointer is non-NULL the call waits for the stream and returns
 * SOLON_E_DECODE / SOLON_E_NUMERIC when a group failed; with all three NULL it is asynchronous and the
 * status is reported by solon_decode_status.
 */
int solon_locate(solon_plan* plan, const float* R, int64_t ldr, const float* f, int32_t* byz_idx, int32_t* n_byz,
                 double* rho_out, void* hip_stream);

/*
 * psi for every group and the sum over groups (Algorithm 1; Lemma 2; Thm. 3):
 *   u[p m + l] = sum_g sum_t T[g][l][t] * R[U_g[t]][p],
 * where U_g holds m honest nodes of group g and T[g] is the inverse of their m x m Vandermonde.
 * Reads q * m rows of R, writes u once.
 *   byz_idx, n_byz  host: the located set to exclude, ascending global indices (byz_idx == NULL with n_byz == 0: the
 *                   empty set); or byz_idx == NULL and n_byz < 0 to use what the preceding solon_locate on this plan left
 *                   on the device (no host round trip)
 *   u               device, d fp32
 */
int solon_decode(solon_plan* plan, const float* R, int64_t ldr, const int32_t* byz_idx, int32_t n_byz, float* u,
                 void* hip_stream);

/*
 * solon_decode fused with the step that follows it in training (Sec. 3.1, "Distributed learning":
 * w_t = w_{t-1} - gamma_t / |S_t| * sum of the gradients): the aggregate u = G 1_P is not written; every coordinate of
 * the parameter vector is read, reduced by step * u[c] and written back by the recombination kernels themselves.
 *   params  device, d fp32, updated in place
 *   step    gamma / |S|: learning rate over the number of per-batch gradients in the sum
 *   R, byz_idx, n_byz as for solon_decode.  Not idempotent: run it once per located round (check solon_decode_status of
 *   the locate call first when the status matters; an update from a failed group is as unspecified as u would be).
 */
int solon_decode_update(solon_plan* plan, const float* R, int64_t ldr, const int32_t* byz_idx, int32_t n_byz, float* params,
                        float step, void* hip_stream);

/*
 * solon_locate followed by solon_decode, in one pass over R (same paper passages; same V, same status, u to the same
 * bar).  The rows for psi are guessed first - by the locator itself, run on the projection of a sample of the columns
 * (128 tiles of 1024 columns at positions hashed from the bits of f, which no sender of R knows) - and the single pass
 * over R produces the exact projections of all P rows together with the recombination of the guessed rows.  The locator
 * then runs on the exact projections as in solon_locate; only if one of the guessed rows turns out to be in V (a node
 * that corrupts a fraction x of its columns escapes the sample with probability (1 - x)^128) the recombination is
 * repeated with the right rows, decided on the device.  When a group's status is not SOLON_OK, u is unspecified.
 * Reads R about once instead of
 * 1 + q m / P times.  Falls back to the two separate passes for m other than 1, 2, 4, unaligned buffers, plans with
 * idle nodes and inputs on which the saved second read of q m rows does not pay for the guess (rows of R below roughly 1.5 GB in all).
 *   R, f            device, as for solon_locate
 *   u               device, d fp32, as for solon_decode
 *   byz_idx, n_byz, rho_out   host or NULL, as for solon_locate; asynchronous when all three are NULL
 */
int solon_locate_decode(solon_plan* plan, const float* R, int64_t ldr, const float* f, float* u, int32_t* byz_idx,
                        int32_t* n_byz, double* rho_out, void* hip_stream);

/*
 * Repetition-code decoder for m = 1 (every honest node of a group sends the group's gradient sum itself; the
 * paper's appendix on the repetition code with its streaming majority vote): u[c] = sum over groups of the value
 * that more than half of the group's nodes sent for coordinate c.  Needs no projection vector and no locate call;
 * it is an independent check of solon_locate + solon_decode at m = 1 and reads R once.
 *   R        device, P x d fp32 (d_c = d when m = 1), row stride ldr
 *   u        device, d fp32
 *   byz_idx  host int32[>= P] or NULL: receives the nodes that differ from their group's majority anywhere
 *   n_byz    host int32* or NULL
 * Returns SOLON_E_INVAL if the plan's m is not 1; SOLON_E_DECODE (through the host outputs or
 * solon_decode_status) if some coordinate of some group has no majority value.  Asynchronous unless a host
 * output pointer is given.
 */
int solon_decode_majority(solon_plan* plan, const float* R, int64_t ldr, float* u, int32_t* byz_idx, int32_t* n_byz,
                          void* hip_stream);

/*
 * solon_locate for callers that cannot allocate device memory or take part in a plan's workspace: code recorded under
 * HIP graph capture in a process that must not call hipMalloc, tight serving loops, harnesses that forbid allocation.
 * Same kernels, same located set and status as solon_locate, but everything they need beyond the caller's buffers (the
 * group tables, the per-tile partial projections, psi's tables) lives in a device array that is part of the library
 * image: about 1.03 MiB held on every GPU the library runs on, until the process ends.  The plan is only read on the
 * host (its own workspace may be missing), no HIP allocation, free, memset or host copy is made, and the call never waits.
 *   R, f      device, as for solon_locate
 *   located   device int32[P] (written: 1 = node in V, 0 = not; idle nodes 0)
 *   status    device int32[q] (written: SOLON_OK / SOLON_E_DECODE / SOLON_E_NUMERIC per group)
 *   rho       device double[P] or NULL (written: the projections)
 * Limits: P <= 128 (SOLON_E_INVAL beyond).  All calls on one GPU share the one array and it keeps the last call's
 * contents: calls that overlap on one GPU (different streams or threads) race and must be ordered by the caller.  Every
 * part a call reads is written by that call first; located[] is cleared by it.
 */
int solon_locate_static(const solon_plan* plan, const float* R, int64_t ldr, const float* f, int32_t* located, int32_t* status,
                        double* rho, void* hip_stream);

/* Waits for hip_stream and returns the status the last solon_locate / solon_decode on this plan left on the
 * device: SOLON_OK, SOLON_E_DECODE or SOLON_E_NUMERIC. */
int solon_decode_status(solon_plan* plan, void* hip_stream);

/* Launch-shape knobs for measurements and tests (process-wide): "encode_phase", "decode_phase" (-1 = choose by size,
 * 0 = flat kernels, 1 = the persistent phase-separated kernels wherever they are legal), "encode_phase_grid",
 * "decode_phase_grid" (cap on the persistent grid, 0 = none), "phase_spin_limit", "project_rows", "project_seg",
 * "encode_blocks", "encode_nt", "encode_force_generic", "decode_blocks", "decode_ch", "decode_force_generic",
 * "fuse" (-1 = solon_locate_decode chooses by size, 0 = always two passes, 1 = one pass wherever legal), "fuse_grid",
 * "fuse_sample" (columns of the sample projection behind the guess), "fuse_sample_leading" (1 = the sample is the leading
 * columns instead of tiles at positions hashed from f: lets a test keep a corruption out of the sample), "fuse_blind_guess"
 * (1 = the guess ignores the sample and takes every node as honest: times the repeated recombination), "fuse_spin_limit", "project_xcd_map",
 * "store_pace_gbps" (rate of the store schedule in the encoder's write phases, GB/s; 0 = stores are not paced),
 * "store_pace_always" (1 = the schedule also runs where the launcher would leave it out: one partly filled phase per group),
 * "majority_rows" (-1 = solon_decode_majority chooses by size, 0 = flat kernels, 1 = the persistent kernel wherever legal),
 * "majority_rows_grid", "solve_basis_table" (0 = the locator wavefront rebuilds the orthonormal polynomials of its consistency test
 * in every call instead of reading the plan's table).
 * Unknown keys are stored and ignored. */
int solon_tune(const char* key, int value);

const char* solon_last_error(void); /* thread-local, valid until the next failing call on this thread */

#ifdef __cplusplus
}
#endif
#endif /* SOLON_H */
