/*
 * fss.h -- C ABI of libfss_mi355: batched function-secret-sharing key generation and
 * evaluation on one AMD MI355X (gfx950), for the two primitives of AriaNN
 * (arXiv 2006.04593): equality 1{x = alpha} (section 3.1, Algorithms 1 and 2) and
 * comparison 1{x <= alpha} (section 3.2, Algorithms 3 and 4), over the ring Z_{2^n},
 * 1 <= n <= 32, with a 128-bit state block (127 seed bits + 1 control bit, appendix C.1).
 *
 * The syntax follows Definition 2.1 of the paper: KeyGen(1^lambda, f) -> (k_0, k_1) and
 * Eval(j, k_j, x) -> the j-th additive share of f(x).  One call handles a batch of
 * independent elements (one key per element), which is the paper's data-parallel "tensor"
 * use of the primitives (section 4.1).  KeyGen's random choices (alpha and the two root
 * seeds, sampled in the initialisation lines of Algorithms 1 and 3) are ARGUMENTS here, so
 * that key generation is a deterministic, auditable function of its inputs.
 *
 * General rules
 *   - Every pointer whose name starts with d_ is DEVICE memory on the current HIP device,
 *     owned by the caller before, during and after the call.  The library allocates no
 *     device memory and keeps no pointer of the caller.  The only state it holds between
 *     calls is per device and never affects results: that its kernels were configured, and
 *     what fss_prepare() describes.
 *   - The FIRST call on a device configures the kernels (one hipDeviceGetAttribute and one
 *     hipFuncSetAttribute per kernel).  Those calls are not allowed while a stream is being
 *     captured into a graph: call fss_prepare() (or any entry point, eagerly) once per device
 *     before capturing.
 *   - Calls only ENQUEUE work on `stream` (a hipStream_t; NULL = the default stream) and
 *     return without waiting; the caller synchronises.  Buffers must stay valid until the
 *     enqueued work has finished.  (The two fss_cmp_eval_streamed* calls block; see there.)
 *   - Return value: FSS_OK (0) or a negative FSS_E* code; nothing aborts or throws.
 *     Arguments are checked on the host before any device work is enqueued, so a call that
 *     fails with FSS_EINVAL or FSS_ELIMIT has no effect.  FSS_ELAUNCH comes from the HIP
 *     runtime; the single-launch entry points have enqueued nothing when they return it, the
 *     streamed ones may have evaluated the chunks before the failure (d_out partly written).
 *     batch == 0 is a successful no-op (pointers may then be NULL).
 *   - Values of alpha, r and x are reduced mod 2^n (high bits ignored).
 *   - Alignment: key buffers 256 bytes; seed arrays 16 bytes; u32 arrays 4 bytes.
 *
 * Key buffer (ONE party's keys for the whole batch; structure of arrays so that the 64
 * lanes of a wavefront read consecutive addresses at every level).  Bp = batch rounded up
 * to a multiple of 64; all integers little-endian; planes follow each other without gaps:
 *
 *   comparison key                                    bytes
 *     alpha_share [Bp]      u32   [[alpha]]_j          4 Bp      (not read by Eval)
 *     seed        [Bp][16]  u8    s_j^(1)              16 Bp
 *     ctrl        [Bp][4]   u32   t_CW^L, t_CW^R,      16 Bp     bit i-1 <-> level i
 *                                 tau_CW^L, tau_CW^R
 *     s_CW        [n][Bp][16] u8                       16 n Bp
 *     sigma_CW    [n][Bp]   u32                        4 n Bp
 *     CW_leaf     [n][Bp]   u32   levels 1..n          4 n Bp
 *     CW_leaf_last[Bp]      u32   level n+1            4 Bp
 *   = 808 bytes per element at n = 32, the paper's n(lambda+2n+4)+lambda+2n bits (3.2.4).
 *
 *   equality key
 *     alpha_share [Bp] u32 | seed [Bp][16] | ctrl [Bp][2] u32 (t_CW^L, t_CW^R) |
 *     s_CW [n][Bp][16] | CW_last [Bp] u32                = 544 bytes per element at n = 32.
 *
 *   The correction-word planes of k_0 and k_1 are identical; the keys differ in seed and
 *   alpha_share.  Elements batch..Bp-1 of every plane are padding (KeyGen writes them
 *   as zeros, so a key buffer is a deterministic function of the arguments; Eval never
 *   reads them).
 *
 * Conventions the paper leaves open, fixed by this library:
 *   - block = 16 bytes in FIPS-197 order; control bit t = bit 0 of byte 0; a seed is a block
 *     with that bit cleared.
 *   - PRG (section 3.1 "Implementation", appendix C.1): G_m(s) = AES128_{k_m}(s) xor s with
 *     fixed keys k_m = 00 01 .. 0e (0f + m - 1), m = 1, 2, 3.  G_1 / G_2 give the left /
 *     right child block (s^b || t^b).  G_3 gives W with sigma^L = LE32(W[0..3]),
 *     sigma^R = LE32(W[4..7]) (mod 2^n), tau^L = W[8] & 1, tau^R = (W[8] >> 1) & 1.
 *   - the map from a seed to Z_{2^n} in the last correction word is LE32(s[12..15]) mod 2^n.
 *   - x[i], alpha[i] for i = 1..n count from the most significant of the n bits; <= is the
 *     unsigned order (section 2, "natural embedding").
 *   - correction words are in the shortened form of the "Implementation" paragraphs: the
 *     seed-sized string of the branch leaving the special path is reused for the branch
 *     staying on it (and, for the sigma lane, the other way round).
 */
#ifndef FSS_MI355_H
#define FSS_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *fss_stream_t; /* hipStream_t */

/* Largest element count of one call (2^40; at 808 bytes per element far beyond any device). */
#define FSS_MAX_BATCH ((size_t)1 << 40)

#define FSS_OK 0
#define FSS_EINVAL (-1)   /* party not in {0,1}; n not in [1,32]; more than FSS_MAX_BATCH elements; NULL or misaligned pointer with batch > 0 */
#define FSS_ELAUNCH (-2)  /* the HIP runtime refused a launch or an attribute; see fss_last_hip_error() */
#define FSS_EDEVICE (-3)  /* current device cannot run the kernels (needs 128 KiB of LDS per workgroup) */
#define FSS_ELIMIT (-4)   /* a size is beyond a fixed limit of the entry point (fss_cmp_eval_streamed_static) */

/* Per-device set-up for the CURRENT device, idempotent and thread-safe: configures the kernels
 * (they need 128 KiB of dynamic LDS) and readies the built-in staging memory of
 * fss_cmp_eval_streamed_static.  Every entry point does its part of this by itself on its first
 * call on a device; calling it explicitly keeps that work out of latency-critical or captured code.
 * FSS_OK, FSS_EDEVICE (the device cannot run the kernels) or FSS_ELAUNCH. */
int fss_prepare(void);

/* Size in bytes of ONE party's key buffer for `batch` elements, padding included
 * (808 * Bp for comparison and 544 * Bp for equality at n = 32).  0 if n is out of range or
 * batch exceeds FSS_MAX_BATCH. */
size_t fss_cmp_key_bytes(int n, size_t batch);
size_t fss_eq_key_bytes(int n, size_t batch);

/* Comparison KeyGen, Algorithm 3 of the paper: for every element e < batch builds the pair
 * (k_0, k_1) of keys for f(x) = 1{x <= alpha[e]}.
 *   d_alpha   [batch] u32   the secret offsets alpha
 *   d_alpha_r [batch] u32   randomness r: [[alpha]]_0 = r, [[alpha]]_1 = alpha - r (mod 2^n)
 *   d_seed0   [batch][16]   party 0's root seed blocks s_0^(1) (bit 0 of byte 0 is ignored)
 *   d_seed1   [batch][16]   party 1's root seed blocks s_1^(1)
 *   d_key0, d_key1          out: fss_cmp_key_bytes(n, batch) bytes each, must not overlap */
int fss_cmp_gen(int n, size_t batch, const uint32_t *d_alpha, const uint32_t *d_alpha_r,
                const uint8_t *d_seed0, const uint8_t *d_seed1, void *d_key0, void *d_key1,
                fss_stream_t stream);

/* Comparison Eval, Algorithm 4: d_out[e] = party `party`'s share of 1{d_x[e] <= alpha[e]},
 * so that d_out(party 0) + d_out(party 1) = 1{x <= alpha} mod 2^n.
 *   d_key  that party's key buffer as written by fss_cmp_gen (same n and batch)
 *   d_x    [batch] u32 public inputs;   d_out [batch] u32 */
int fss_cmp_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_x,
                 uint32_t *d_out, fss_stream_t stream);

/* Equality KeyGen / Eval, Algorithms 1 and 2; same argument meaning, f(x) = 1{x = alpha},
 * key buffers of fss_eq_key_bytes(n, batch) bytes. */
int fss_eq_gen(int n, size_t batch, const uint32_t *d_alpha, const uint32_t *d_alpha_r,
               const uint8_t *d_seed0, const uint8_t *d_seed1, void *d_key0, void *d_key1,
               fss_stream_t stream);
int fss_eq_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_x,
                uint32_t *d_out, fss_stream_t stream);

/* ---- the steps around the comparison: Sign protocol and ReLU ---------------------------
 *
 * Sign protocol, Algorithm 5 of the paper, for shared inputs [[y]]: each party publishes
 * [[y]]_j + [[alpha]]_j (fss_sign_mask; [[alpha]]_j is the first plane of its key), both add
 * the two published vectors to x = y + alpha and evaluate the comparison key on it
 * (fss_sign_eval, reveal fused into the evaluation kernel).  The result is a share of
 * 1{y <= 0} except with probability |y| / 2^n (section 3.2.2).
 *
 * ReLU, section 4.2: ReLU(y) = y . (1 - 1{y <= 0}), the comparison followed by ONE pointwise
 * product of shared values with a multiplication triple ([[a]], [[b]], [[c]] = [[a.b]]) as in
 * the paper's MatMul paragraph; 2 rounds, 3 values per element (Table 2).
 *   round 1: publish fss_sign_mask's output;
 *   round 2: fss_relu_open evaluates the comparison and directly forms the party's messages
 *            delta_j = [[y]]_j - [[a]]_j and eps_j = ([j = 0] - [[1{y<=0}]]_j) - [[b]]_j;
 *   then     fss_relu_finish: [[ReLU(y)]]_j = delta.[[b]]_j + eps.[[a]]_j + [[c]]_j (+ delta.eps
 *            for party 0), delta = delta_0 + delta_1, eps = eps_0 + eps_1.
 * All arrays are [batch] u32 device arrays of that party unless they carry the other party's
 * index (published values).  The exchange between the parties is the caller's business. */
int fss_sign_mask(int n, size_t batch, const void *d_key, const uint32_t *d_y_share, uint32_t *d_masked,
                  fss_stream_t stream);
int fss_sign_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_masked0,
                  const uint32_t *d_masked1, uint32_t *d_out, fss_stream_t stream);
int fss_relu_open(int party, int n, size_t batch, const void *d_key, const uint32_t *d_masked0,
                  const uint32_t *d_masked1, const uint32_t *d_y_share, const uint32_t *d_tri_a,
                  const uint32_t *d_tri_b, uint32_t *d_delta, uint32_t *d_eps, fss_stream_t stream);
int fss_relu_finish(int party, int n, size_t batch, const uint32_t *d_delta0, const uint32_t *d_delta1,
                    const uint32_t *d_eps0, const uint32_t *d_eps1, const uint32_t *d_tri_a,
                    const uint32_t *d_tri_b, const uint32_t *d_tri_c, uint32_t *d_out, fss_stream_t stream);

/* ---- Argmax (Algorithm 6) and MaxPool (Algorithm 7) as compositions ----------------------
 *
 * Equality on shared inputs (wrapper lines of Algorithm 2): fss_eq_mask publishes
 * [[alpha]]_j + [[y]]_j from an equality key; fss_eq_masked_eval adds the two published vectors
 * and evaluates: a share of 1{y = 0}.
 *
 * Argmax of `rows` vectors of m shared values, 2 rounds:
 *   fss_argmax_diff_mask   masked shares of x_i - x_j for every ordered pair (j, i), i != j, under
 *                          comparison keys for rows*m*(m-1) elements; element ((r m + j)(m-1) + t)
 *                          holds i = t for t < j and i = t + 1 otherwise            -> round 1
 *   fss_sign_eval          on the revealed differences: shares of 1{x_i <= x_j}
 *   fss_argmax_count_mask  [[s_j]] = sum of the m-1 shares of (r, j); masked share of s_j - (m-1)
 *                          under equality keys for rows*m elements                  -> round 2
 *   fss_eq_masked_eval     shares of 1{s_j = m-1}: the argmax in one-hot form (all maxima on ties)
 * MaxPool (k x k windows, stride s, no padding) of a [channels][h][w] tensor of shares, 3 rounds:
 *   fss_maxpool_unroll     one row of k*k shares per window, windows in (channel, y, x) order
 *   Argmax of the rows (m = k*k), then the inner product of each row with its one-hot vector:
 *   fss_mul_open           delta_j = [[u]]_j - [[a]]_j, eps_j = [[v]]_j - [[b]]_j   -> round 3
 *   fss_dot_finish         [[y_r]]_j = sum over the row of delta.[[b]]_j + eps.[[a]]_j + [[c]]_j
 *                          (+ delta.eps for party 0)
 * All arrays are u32 device arrays; sizes follow from rows, m, channels, h, w, k, s. */
int fss_eq_mask(int n, size_t batch, const void *d_key, const uint32_t *d_y_share, uint32_t *d_masked,
                fss_stream_t stream);
int fss_eq_masked_eval(int party, int n, size_t batch, const void *d_key, const uint32_t *d_masked0,
                       const uint32_t *d_masked1, uint32_t *d_out, fss_stream_t stream);
int fss_argmax_diff_mask(int n, size_t rows, int m, const void *d_cmp_key, const uint32_t *d_x_share,
                         uint32_t *d_masked, fss_stream_t stream);
int fss_argmax_count_mask(int party, int n, size_t rows, int m, const uint32_t *d_w_share,
                          const void *d_eq_key, uint32_t *d_masked, fss_stream_t stream);
int fss_maxpool_unroll(size_t channels, int h, int w, int k, int s, const uint32_t *d_x_share,
                       uint32_t *d_rows, fss_stream_t stream);
int fss_mul_open(int n, size_t count, const uint32_t *d_u_share, const uint32_t *d_v_share,
                 const uint32_t *d_tri_a, const uint32_t *d_tri_b, uint32_t *d_delta, uint32_t *d_eps,
                 fss_stream_t stream);
int fss_dot_finish(int party, int n, size_t rows, int m, const uint32_t *d_delta0, const uint32_t *d_delta1,
                   const uint32_t *d_eps0, const uint32_t *d_eps1, const uint32_t *d_tri_a,
                   const uint32_t *d_tri_b, const uint32_t *d_tri_c, uint32_t *d_out, fss_stream_t stream);

/* ---- keys kept in host memory, imported during the online phase --------------------------
 *
 * The paper notes (section 5.2) that device memory for keys limits the batch size and that
 * keeping keys on the host and importing them online would lift that.  Chunked host layout:
 * the batch is cut into consecutive chunks of `chunk` elements (the last may be shorter);
 * chunk c is an ordinary key buffer for its own elements, fss_cmp_key_bytes(n, len_c) bytes,
 * and the chunks follow each other without gaps in `h_key_chunks` (PINNED host memory,
 * allocated by the caller with hipHostMalloc or torch's pin_memory; pageable memory works but
 * serialises the copies).  fss_cmp_chunked_key_bytes gives the total size.
 *
 * fss_cmp_eval_streamed copies chunk c+1 host-to-device on `copy_stream` into one half of
 * `d_staging` while chunk c is evaluated on `stream` out of the other half, ordering the two
 * with events it creates and destroys inside the call.  d_staging: device memory,
 * 2 * fss_cmp_key_bytes(n, chunk) bytes, 256-byte aligned.  chunk must be a multiple of 64.
 * Unlike the other entry points this one BLOCKS until the last chunk has been evaluated (it has
 * to recycle the staging halves), and `copy_stream` must differ from `stream`.  Results are
 * identical to fss_cmp_eval on the same keys.  The rate is bounded by the host link:
 * 808 bytes per element at n = 32. */
size_t fss_cmp_chunked_key_bytes(int n, size_t batch, size_t chunk);
int fss_cmp_eval_streamed(int party, int n, size_t batch, size_t chunk, const void *h_key_chunks,
                          const uint32_t *d_x, uint32_t *d_out, void *d_staging,
                          fss_stream_t copy_stream, fss_stream_t stream);

/* For callers that cannot allocate device memory (code under HIP graph capture elsewhere in the
 * process, tight serving loops, harnesses that forbid hipMalloc): fss_cmp_eval_streamed with the
 * two staging halves taken from a fixed array inside the library instead of `d_staging`, and with
 * events made once per device instead of per call.  Same arguments otherwise, same results.
 *   - Limit: 2 * fss_cmp_key_bytes(n, chunk) <= fss_static_staging_bytes() (32 MiB: chunk up to
 *     20,736 elements at n = 32); beyond it the call returns FSS_ELIMIT and does nothing.
 *   - After the per-device set-up the call allocates nothing: no hipMalloc/hipFree, no event or
 *     stream creation -- only hipMemcpyAsync from the caller's PINNED host buffer, event
 *     records/waits, kernel launches and two stream synchronisations.  The set-up (the array's
 *     device address, four events, kernel attributes) happens in fss_prepare(), or else in the
 *     first call on a device; call fss_prepare() up front to keep even that out of the path.
 *   - The array is one per GPU and shared by every call on that GPU, for the life of the process:
 *     calls that overlap in time on one GPU (from several threads or stream pairs) race on it and
 *     must be serialised by the caller.  Nothing in it needs clearing between calls: every byte
 *     a kernel reads has been overwritten by that call's own copies first.
 *   - Like fss_cmp_eval_streamed it blocks until the last chunk has been evaluated. */
size_t fss_static_staging_bytes(void);
int fss_cmp_eval_streamed_static(int party, int n, size_t batch, size_t chunk, const void *h_key_chunks,
                                 const uint32_t *d_x, uint32_t *d_out, fss_stream_t copy_stream,
                                 fss_stream_t stream);

/* Register layouts.  The KeyGen and Eval kernels walk an element in one of two layouts with identical
 * results (keys and shares agree byte for byte): one lane per element (highest throughput) and four
 * lanes per element (a quarter of the dependent work per wavefront and four times the wavefronts:
 * lower latency while there is too little work to fill the device).  The entry points pick by batch
 * size: below fss_quad_layout_below() elements (512 per compute unit) everything runs four lanes per
 * element; from there on, one lane per element in rows of 64 elements per compute unit (16 rows =
 * 2 * fss_quad_layout_below() elements make a full pass), and what is left after the last full pass
 * -- if it is shorter than fss_quad_layout_below() -- as well as the last partial row run four lanes
 * per element inside the same launch.  Up to fss_quad_layout_below() / 4 elements, KeyGen and the
 * comparison Eval spread an element over eight lanes (KeyGen one quad per party, Eval one quad per
 * PRG block of a level).
 * fss_quad_layout_below() returns that size for the current device, or 0 if the device cannot be
 * queried.
 * The kernels change the priority of their own wavefronts (s_setprio) while they run, so that the
 * wavefronts sharing a SIMD advance together; kernels of other streams running beside them on the
 * same compute units compete with priorities between 0 and 3. */
size_t fss_quad_layout_below(void);

/* Measurement aid (no part of the method): the clock the chip sustains.  fss_clock_probe enqueues
 * ONE wavefront that sleeps for `iterations` (1 .. 2^20) x 8128 shader clocks -- about 3.4 us each --
 * and then writes d_ticks[0] = shader clocks elapsed, d_ticks[1] = ticks of the constant-rate wall
 * clock elapsed (two u64, device memory, 8-byte aligned).  Launched on a second stream beside the
 * kernels of interest, shader clocks / wall ticks x fss_wall_clock_khz() is the clock in kHz under
 * that load.  fss_wall_clock_khz: rate of the wall clock of the current device, 0 if unknown. */
int fss_clock_probe(uint64_t *d_ticks, uint32_t iterations, fss_stream_t stream);
int fss_wall_clock_khz(void);

/* Text for a return code (static storage, never NULL). */
const char *fss_strerror(int code);

/* The hipError_t value behind the most recent FSS_ELAUNCH / FSS_EDEVICE on this thread. */
int fss_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FSS_MI355_H */
