/*
 * ws_synapse.h -- C ABI of the Topological Synapse hot path for AMD MI355X (gfx950).
 *
 * The Topological Synapse (Warp-Cortex, Sec. 3.3) is a shared buffer holding k << L
 * "landmark" rows of the main agent's KV cache; side agents attend over those k rows
 * instead of the whole context.  Landmarks are chosen per KV head by treating the L
 * cached keys as a point cloud and scoring each point by a hybrid of geometric
 * coverage and inverse kernel density (Sec. 3.3, "Hybrid Density-Coverage Sampler";
 * Sec. 2, first paragraph).  The four entry points below are the four stages of that
 * path: density -> select -> gather -> attend.
 *
 * Conventions shared by every entry point
 *   - Pointers marked "dev" are device (HBM) pointers; "host" are host pointers.
 *   - Tensors are dense row-major with the head dimension d innermost.  "H" is
 *     whatever the caller flattens into independent KV heads (layers x heads).
 *   - dtype selects the element type of K, V, Q, Ks, Vs: WS_F32 (4 bytes) or WS_BF16
 *     (2 bytes, upper half of an IEEE float).  Accumulation is always fp32.
 *   - K, V, Q, Ks, Vs must be 16-byte aligned; d must be 64 or 128.
 *   - The caller owns every buffer, including the workspace (size from
 *     ws_synapse_workspace_bytes, 256-byte aligned).  The library allocates nothing,
 *     keeps no state between calls, reads no environment variable and never synchronises
 *     the host (ws_synapse_select_failed and ws_synapse_density_check, which read a flag back, are
 *     the exceptions):
 *     all work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null
 *     stream), so a caller can run the producer on one stream and the agents on others
 *     (Sec. 3.1).  Two calls that share a workspace must be ordered by the caller.
 *   - Errors are return codes only.  Arguments are validated on the host before any
 *     launch; on an error nothing has been enqueued.  Non-finite inputs give
 *     undefined results, not errors.
 */
#ifndef WS_SYNAPSE_H
#define WS_SYNAPSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WS_OK = 0,
    WS_ERR_INVALID_ARG = 1,  /* NULL pointer, size < 1, k > L, alpha outside [0,1], sigma <= 0, misalignment */
    WS_ERR_UNSUPPORTED = 2,  /* d not in {64,128}, unknown dtype, L >= 2^24, a kernel that does not fit was named */
    WS_ERR_WORKSPACE = 3,    /* workspace NULL, misaligned or smaller than ws_synapse_workspace_bytes() */
    WS_ERR_HIP = 4,          /* a HIP call or kernel launch failed; see hipGetLastError() */
    WS_ERR_TOO_LARGE = 5,    /* ws_synapse_select_static only: the sizes need more than its fixed scratch */
    WS_STATUS_INT_RANGE = 0x7fffffff   /* not a status: gives the type the range of int (see below) */
} ws_status;

/* Every enum of this header ends in such an enumerator, so that any int a caller passes is a value of the
 * type and reaches the library's own checks (an unknown dtype or op is answered with an error code). */
typedef enum { WS_F32 = 0, WS_BF16 = 1, WS_DTYPE_INT_RANGE = 0x7fffffff } ws_dtype;

typedef enum {
    WS_OP_DENSITY = 0, WS_OP_SELECT = 1, WS_OP_GATHER = 2,
    WS_OP_ATTEND = 3,          /* H = KV heads, Hq = query heads (a multiple of H), k, N; L is not used */
    WS_OP_ATTENTION_MASS = 4,  /* H = G*Hkv heads, Hq = query heads per group times G */
    WS_OP_DENSITY_APPEND = 5,  /* k = m appended rows */
    WS_OP_INJECT = 6,          /* k = m injected rows */
    WS_OP_INT_RANGE = 0x7fffffff
} ws_op;

typedef void *ws_stream; /* hipStream_t */

/*
 * Gaussian kernel density of every key against all keys of the same head
 * (the "inverse kernel density" ingredient of the hybrid score, Sec. 2 and Sec. 3.3):
 *     rho[h,i] = (1/L) * sum_{j<L} exp(-||K[h,i]-K[h,j]||^2 / (2 sigma[h]^2)),  j = i included,
 * no Gaussian normalising constant, so 1/L <= rho <= 1.
 *   K          dev  [H,L,d] keys, dtype `dt`
 *   sigma_host host [H] bandwidths, each finite and > 0 (read before the call returns); a bandwidth above
 *              about 7e13 (where every kernel value is 1 to fp32 precision anyway) is WS_ERR_UNSUPPORTED
 *   rho        dev  [H,L] fp32, written
 *
 * Accuracy.  The squared distances come from a Gram product on the matrix cores, so one kernel term
 * carries a relative error of about 2^-23 * mean|k - c|^2 / sigma^2, where c is a reference point the
 * library subtracts first: per head and coordinate the mid-range of the keys, wherever the differences
 * k - c are exact in the keys' own format (a cloud sitting at a common offset, as real key caches do,
 * is moved back to the origin at no loss; bf16 keys only).  The errors of different terms are independent
 * and average down in the sum; with the bandwidth comparable to the cloud's spread (sigma^2 = tr(Cov)/16:
 * estimate 2e-6) rho is within 5e-5 (bf16) / 1e-5 (fp32) of the exact value.  The estimate grows as the
 * bandwidth shrinks below the spread and for offsets that cannot be removed exactly; every call writes it
 * per head to the workspace and raises a flag when it exceeds 2e-5 (ws_synapse_density_check).  An isolated
 * key's self term is exact whatever the estimate.  fp32 keys are swept in place (no translation).
 */
ws_status ws_synapse_density(const void *K, ws_dtype dt, int H, int L, int d,
                             const float *sigma_host, float *rho,
                             void *workspace, size_t workspace_bytes, ws_stream stream);

/* Accuracy report of the last ws_synapse_density enqueued on `stream` with this workspace (the first 256
 * bytes of the workspace are the flag block, int32 flag at offset 0; H floats of estimates follow).  Waits
 * for the stream (like ws_synapse_select_failed, this call synchronises the host), then writes to *flagged
 * 1 if some head's estimated relative error per kernel term exceeds 2e-5, else 0, and, if err_est is not
 * NULL, the H estimates (host array). */
ws_status ws_synapse_density_check(const void *workspace, int H, ws_stream stream, int *flagged, float *err_est);

/* Which sweep ws_synapse_density runs for these sizes: 1 = the symmetric sweep (every unordered pair once),
 * 0 = the full sweep.  For reports and profiles. */
int ws_synapse_density_is_symmetric(ws_dtype dt, int L, int d);

/*
 * Greedy landmark choice per head (Sec. 3.3: coverage in the Hausdorff sense balanced
 * against inverse density; k landmarks).  With u_i = min_j(rho_j)/rho_i, D_i the Euclidean
 * distance from key i to the nearest landmark chosen so far and D_max the current maximum
 * of D over the keys not yet chosen, step t picks
 *     argmax_i  alpha * D_i/D_max + (1-alpha) * u_i      over keys not yet chosen,
 * lowest index on ties; D_max == 0 makes the first term 0.  With no landmark yet the first
 * term is 1 for every key, so step 0 picks argmax u (alpha < 1) or index 0 (alpha == 1).
 *   K         dev [H,L,d];  rho dev [H,L] fp32 (from ws_synapse_density)
 *   k         landmarks per head, 1 <= k <= L;  alpha in [0,1] (1 = coverage only)
 *   idx       dev [H,k] int32, written in pick order
 *   score_out dev [H,k] fp32 winning score per step, or NULL
 *
 * Two kernels implement this call: one keeps a head's keys resident in registers and LDS for all
 * k steps (bf16 keys, heads that fit on chip), one streams them from memory every step (any size).
 * ws_synapse_select lets the library pick; ws_synapse_select_with names one.
 *
 * Co-residency contract.  Both kernels are persistent: the workgroups that share a head exchange
 * their partial maxima every step and wait for each other, so the WHOLE grid has to be resident on
 * the device at once.  The launch is sized from the current device (its compute-unit count and the
 * number of workgroups of the kernel a compute unit holds, both asked of the runtime at every call),
 * which guarantees this when the selection has the device to itself.  The paper runs the producer
 * beside other streams (Sec. 3.1, Sec. 4); work on other streams that holds compute units while a
 * selection starts (a second selection in particular: AT MOST ONE SELECTION MAY BE IN FLIGHT PER
 * DEVICE) can keep part of the grid from becoming resident.  Short kernels only delay it: every wait
 * is a bounded spin of a few seconds.  If a wait does expire the kernel gives up cleanly: it sets the
 * failure flag, writes -1 into the entries of idx it still owes for the affected heads, and drains.
 * The call has long returned WS_OK by then, so the flag is the only report:
 *   - the first 256 bytes of the selection workspace are the flag block; the int32 at offset 0 is 0
 *     after a complete selection and 1 after one that gave up (it is reset by every call);
 *   - ws_synapse_select_failed copies it to the host after synchronising the stream;
 *   - ws_synapse_gather clamps a -1 to row 0 rather than following it, so a caller that skips the
 *     check gets a wrong synapse, never a fault.
 */
ws_status ws_synapse_select(const void *K, ws_dtype dt, int H, int L, int d,
                            const float *rho, int k, float alpha,
                            int32_t *idx, float *score_out,
                            void *workspace, size_t workspace_bytes, ws_stream stream);

/* The same step with the kernel named by the caller (tests and profiles; results are identical).
 * WS_SELECT_RESIDENT returns WS_ERR_UNSUPPORTED when no resident instance fits the sizes on the
 * current device (fp32 keys, heads too long to sit on chip). */
typedef enum {
    WS_SELECT_AUTO = 0, WS_SELECT_STREAMING = 1, WS_SELECT_RESIDENT = 2, WS_SELECT_INT_RANGE = 0x7fffffff
} ws_select_kernel;
ws_status ws_synapse_select_with(ws_select_kernel which, const void *K, ws_dtype dt, int H, int L, int d,
                                 const float *rho, int k, float alpha,
                                 int32_t *idx, float *score_out,
                                 void *workspace, size_t workspace_bytes, ws_stream stream);

/*
 * ws_synapse_select for callers that cannot allocate and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * same results as ws_synapse_select, but the scratch the kernels need (failure flag, exchange slots, and
 * the streaming kernel's distance / inverse-density slabs) lives in a fixed array inside the library's
 * device image: 256 bytes + 1 MiB + 4 MiB = 5 243 136 bytes per device, held until the process ends.
 * The call allocates nothing (no hipMalloc, no hipFree, no allocating library routine) and clears what it
 * needs with a small kernel on `stream`.
 *   - Sizes whose scratch does not fit are refused with WS_ERR_TOO_LARGE before anything is enqueued.  The
 *     on-chip kernel (bf16 heads that fit the chip: every size it serves) always fits; the streaming kernel
 *     runs as many heads at once as fit 4 MiB of slabs (8 bytes per key and head in flight), and a single
 *     head must fit: L <= 524 288.
 *   - Every call on a device shares that device's array, which keeps the last call's contents: calls that
 *     overlap on one device (two streams, two threads) race.  Order them, as with a shared workspace; the
 *     one-selection-in-flight rule above applies anyway.
 *   - ws_synapse_select_failed(NULL, stream, &failed) reads this array's failure flag on the current device.
 */
ws_status ws_synapse_select_static(const void *K, ws_dtype dt, int H, int L, int d,
                                   const float *rho, int k, float alpha,
                                   int32_t *idx, float *score_out, ws_stream stream);

/* Did the last selection enqueued on `stream` with this workspace give up (see the co-residency
 * contract above)?  Waits for the stream, then writes 0 or 1 to *failed (host).  workspace == NULL
 * means the fixed scratch of ws_synapse_select_static on the current device.  This call synchronises
 * the host. */
ws_status ws_synapse_select_failed(const void *workspace, ws_stream stream, int *failed);

/* How a selection of these sizes is launched: which kernel, how many heads are in flight at once,
 * how many workgroups share a head.  compute_units = 0 and workgroups_per_cu = 0 ask the current
 * device (256 and the kernels' design value where none is visible); other values answer for a
 * device of that shape (capacity planning, tests).  heads_in_flight * workgroups_per_head never
 * exceeds compute_units * workgroups per unit.  WS_ERR_UNSUPPORTED: `which` names the resident
 * kernel and no instance fits. */
typedef struct {
    int resident;             /* 1 = keys resident on chip, 0 = streaming */
    int heads_in_flight;
    int workgroups_per_head;
    int threads;              /* per workgroup */
    int rows_in_registers;    /* resident kernel: key rows per lane held in registers ... */
    int rows_in_lds;          /* ... and in LDS */
    int compute_units;        /* the device shape the plan was made for */
} ws_select_plan;
ws_status ws_synapse_select_plan(ws_select_kernel which, ws_dtype dt, int H, int L, int d,
                                 int compute_units, int workgroups_per_cu, ws_select_plan *plan);

/*
 * Fill the synapse buffer (Sec. 3.3, "a shared memory buffer containing only Landmarks"):
 *     Ks[h,t,:] = K[h, idx[h,t], :],  Vs[h,t,:] = V[h, idx[h,t], :]     (bit copies, pick order)
 *   K, V dev [H,L,d];  idx dev [H,k] with 0 <= idx < L;  Ks, Vs dev [H,k,d], written.
 * An index outside [0,L) is clamped into range rather than followed.
 */
ws_status ws_synapse_gather(const void *K, const void *V, ws_dtype dt, int H, int L, int d,
                            const int32_t *idx, int k, void *Ks, void *Vs, ws_stream stream);

/*
 * N agents' decode queries attend over the k landmarks instead of the L-row context
 * (Sec. 3.3 gives the 1/sqrt(d_k) scale; Sec. 4 states the O(k) cost):
 *     O[n,q,:] = softmax_t( scale * Q[n,q,:] . Ks[q/g,t,:] ) . Vs[q/g,:,:],   g = Hq/Hkv, t < k
 * no mask (every landmark is past context); all agents read the same synapse.
 *   Q dev [N,Hq,d];  Ks, Vs dev [Hkv,k,d];  Hq % Hkv == 0;  scale <= 0 means 1/sqrt(d)
 *   O dev [N,Hq,d] fp32, written.  workspace may be NULL when the reported size is 0 (it is, unless few heads
 *   meet many landmarks: then the landmark range is split over several workgroups per head, whose partial rows
 *   pass through the workspace and are merged by a second small kernel; the split depends on the sizes only).
 */
ws_status ws_synapse_attend(const void *Q, const void *Ks, const void *Vs, ws_dtype dt,
                            int N, int Hq, int Hkv, int k, int d, float scale, float *O,
                            void *workspace, size_t workspace_bytes, ws_stream stream);

/*
 * Gather and attend in one pass (Sec. 3.3: the synapse holds the landmark rows only; Sec. 4: O(k) per query): the
 * same attention read straight from the chosen rows of the cache, for callers that do not need the synapse as a
 * buffer of its own,
 *     O[n,q,:] = softmax_t( scale * Q[n,q,:] . K[q/g, idx[q/g,t], :] ) . V[q/g, idx[q/g,:], :],   t < k.
 * The result is bit-identical to ws_synapse_gather followed by ws_synapse_attend.
 *   Q dev [N,Hq,d];  K, V dev [Hkv,L,d];  idx dev [Hkv,k], an index outside [0,L) is clamped into range;
 *   O dev [N,Hq,d] fp32, written;  workspace as for ws_synapse_attend (same size, WS_OP_ATTEND).
 *   L * d * sizeof(element) must stay below 2^32 (WS_ERR_UNSUPPORTED otherwise).
 */
ws_status ws_synapse_attend_indexed(const void *Q, const void *K, const void *V, const int32_t *idx,
                                    ws_dtype dt, int N, int Hq, int Hkv, int L, int k, int d, float scale,
                                    float *O, void *workspace, size_t workspace_bytes, ws_stream stream);

/* ------------------------------------------------------------------------------------------
 * Steps next to the hot path.
 * ------------------------------------------------------------------------------------------ */

/*
 * Attention-mass density proxy (Sec. 3.3, "Attention Score Summation"): the density ingredient
 * taken from the main agent's current query instead of a kernel density over the keys, at
 * O(L d) per head instead of O(L^2 d).  Heads come in G groups (layers) of Hkv KV heads and Hq
 * query heads, Hq % Hkv == 0, query head q of a group reading KV head q / (Hq/Hkv).  Per group,
 *     A_i = sum_{q < Hq} softmax_i( scale * Q[q,:] . K[kv(q), i, :] ),   softmax over the L tokens,
 * so sum_i A_i = Hq.  The passage uses A as the INVERSE density: with as_density != 0 the value
 * written is 1 / max(A_i, 1e-30), which ws_synapse_select takes in place of rho (u_i = A_i/A_max);
 * with as_density == 0 it is A_i itself.
 *   K   dev [G*Hkv, L, d];  Q dev [G*Hq, d] (one query token per head), both dtype `dt`
 *   out dev [G*Hkv, L] fp32: every KV head of a group receives the group's values
 *   Hq <= 128 per group, Hq/Hkv <= 8;  scale <= 0 means 1/sqrt(d)
 */
ws_status ws_synapse_attention_mass(const void *K, const void *Q, ws_dtype dt, int G, int Hkv, int Hq,
                                    int L, int d, float scale, int as_density, float *out,
                                    void *workspace, size_t workspace_bytes, ws_stream stream);

/*
 * Density refresh after the context has grown by m rows (Sec. 4: the main stream re-extracts
 * landmarks inside its decode loop).  K holds the L rows AFTER the append, the new ones last;
 * rho_old is the density of the first L-m rows (from ws_synapse_density or an earlier refresh,
 * same sigma).  L*rho is a plain sum of kernel values, so
 *     rho_new[j] = ((L-m) * rho_old[j] + sum_{r<m} w(j, L-m+r)) / L            j < L-m
 *     rho_new[L-m+r] = (sum_{j<L} w(j, L-m+r)) / L                             r < m
 * with w(i,j) = exp(-||K_i-K_j||^2 / (2 sigma^2)); distances by direct differences in fp32.
 * Cost O(L m d) per head.  Each refresh adds fp32 rounding to the old entries; a full
 * ws_synapse_density at every re-selection sheds it.
 *   K dev [H,L,d];  1 <= m <= 32, m < L;  sigma_host host [H];  rho_old dev [H,L-m];  rho_new dev [H,L]
 */
ws_status ws_synapse_density_append(const void *K, ws_dtype dt, int H, int L, int d, int m,
                                    const float *sigma_host, const float *rho_old, float *rho_new,
                                    void *workspace, size_t workspace_bytes, ws_stream stream);

/*
 * Validation gate (Sec. 3.5 and its equation): cosine similarity between the main agent's hidden
 * state and each side agent's thought vector; a thought passes when the score reaches theta.
 *     score[n] = (h . T[n]) / (||h|| ||T[n]||)   (0 when either norm is 0),  accept[n] = score[n] >= theta
 *   h_main dev [dm];  T dev [N,dm], dtype `dt`, 4-byte aligned rows at least (16-byte aligned rows
 *   are read with wide loads);  score dev [N] fp32;  accept dev [N] int32 (1 = passes)
 * The decision is taken on the fp32 score that is written.
 */
ws_status ws_synapse_gate(const void *h_main, const void *T, ws_dtype dt, int N, int dm, float theta,
                          float *score, int32_t *accept, ws_stream stream);

/*
 * Referential injection, cache side (Sec. 3.6): m key/value rows computed elsewhere for a side
 * agent's thought join the main agent's cache in place.  The keys are rotated by RoPE at
 * caller-given virtual positions, the values are copied; rows 0..L-1 are not touched.
 *     pairs (c, c+d/2), angle a = pos[r] * base^(-2c/d):
 *     Kc[h,L+r,c] = x_c cos a - x_{c+d/2} sin a,   Kc[h,L+r,c+d/2] = x_{c+d/2} cos a + x_c sin a
 * Angles are formed in float64 and reduced before the fp32 sine/cosine, so positions up to 2^31
 * keep full accuracy.
 *   Kc, Vc dev [H,Lcap,d] caches with L rows in use, L + m <= Lcap
 *   Knew, Vnew dev [H,m,d] un-rotated rows;  pos dev [m] int32;  base > 0 (e.g. 1e6)
 *   workspace: cos/sin table of the m positions
 */
ws_status ws_synapse_inject(void *Kc, void *Vc, ws_dtype dt, int H, int Lcap, int d, int L,
                            const void *Knew, const void *Vnew, int m, const int32_t *pos, float base,
                            void *workspace, size_t workspace_bytes, ws_stream stream);

/* Which selection kernel ws_synapse_select would run for these sizes on the current device:
 * 1 = keys resident on chip, 0 = streaming.  For reports and profiles. */
int ws_synapse_select_is_resident(ws_dtype dt, int H, int L, int d);

/* Bytes of workspace the given operation needs for these sizes (0 if none).  Arguments an
 * operation does not use are ignored.  Returns (size_t)-1 for unsupported sizes. */
size_t ws_synapse_workspace_bytes(ws_op op, ws_dtype dt, int H, int L, int d, int k, int N, int Hq);

/* Static, NUL-terminated description of a status code. */
const char *ws_status_string(ws_status s);

#ifdef __cplusplus
}
#endif
#endif /* WS_SYNAPSE_H */
