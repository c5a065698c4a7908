/*
 * perq.h -- C ABI of the MI355X (gfx950) PeRQ online activation path.
 *
 * The path, in the paper's notation (Section 1, Notation; Figure 2):
 *
 *     X[T,d] (bf16)  --P-->  XP  --R~ = I_n (x) R-->  XP R~  --Q-->  packed 4-bit codes + scales
 *
 * P  is a channel permutation, (XP)_i = X_{perm[i]};  R is the normalised b x b Sylvester
 * Hadamard matrix (entries +-1/sqrt(b)), d = n*b;  Q is either the symmetric INT4 quantizer
 * with one step per token (Section 3; Appendix B Eq. 4 with z = 0) or MXFP4 (Appendix B Eq. 5:
 * e2m1 elements, one power-of-two scale per 32 contiguous outputs).  The permutation comes
 * from Algorithm 1 (mass diffusion), whose only data dependence is the per-channel mean
 * magnitude a_i = (1/m) sum_k |X_i^(k)|.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device, "host" pointers are
 *     ordinary host memory.  Every buffer is owned by the caller; the library allocates nothing
 *     and frees nothing.  Its only state on a device is a table of scheduling counters (64 sets of
 *     32, in device memory of the library's own) for the run-time row schedule of its main kernel.
 *     Every launch leaves its counters at zero, and a set belongs to one stream: the first 64
 *     streams per device that reach that kernel get a set each and keep it for the life of the
 *     process.  Launches of one stream never run side by side, so no two launches draw from one
 *     set at the same time, however many streams overlap.  A launch from a 65th stream, and any
 *     launch that is being captured into a graph (a graph can be replayed beside anything), takes
 *     a fixed split of the rows instead (same results; the schedule only balances run time,
 *     about 10 % on the largest shapes).  See perq_schedule_set / perq_reset_schedule.
 *   - bf16 tensors are passed as uint16_t bit patterns, row-major, leading dimension in
 *     elements.
 *   - Device entry points enqueue on `hip_stream` (a hipStream_t, NULL = default stream) and
 *     return without synchronising; outputs are valid once the stream has been synchronised.
 *   - Every entry point returns a perq_status_t; nothing throws or aborts.  Arguments are
 *     checked on the host before any launch.  Contents of `perm` are NOT checked on the
 *     device: a perm that is not a bijection on [0,d) gives undefined output values (reads
 *     stay inside the row only if every entry is in [0,d); validate with perq_perm_validate).
 *   - Non-finite inputs give unspecified output values but no fault.
 */
#ifndef PERQ_H
#define PERQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PERQ_OK = 0,
    PERQ_ERR_INVALID_ARG = 1,  /* null pointer, bad size, b not a power of two in [16,d], ... */
    PERQ_ERR_UNSUPPORTED = 2,  /* valid problem the kernels do not cover (alignment, d too large) */
    PERQ_ERR_LAUNCH = 3,       /* HIP reported an error at launch */
    PERQ_ERR_INTERNAL = 4      /* a consistency check of the library's own failed (never expected) */
} perq_status_t;

typedef enum {
    PERQ_FMT_INT4_SYM_TOKEN = 0,  /* codes in [-7,7] as two's-complement nibbles; float scale per token */
    PERQ_FMT_MXFP4 = 1,           /* e2m1 nibbles (sign|exp2|mant1); e8m0 byte per 32 outputs */
    /* Appendix B, INT4 paragraph (the activation quantizer of the paper's INT4 results): per token
     * step s = (max - min)/15 and integer zero point z = rne(min/s); codes rne(y/s) - z clipped to
     * [0,15] as unsigned nibbles; a code stands for s*(code + z).  scales: float [T][2] = (s, z),
     * 8-byte aligned.  A constant row gives s = 0, z = 0, codes 0. */
    PERQ_FMT_INT4_ASYM_TOKEN = 2,
    /* Appendix B, (MX)FP4 paragraph: e2m1 nibbles with one real scale per token,
     * s = max|y| / 6 (6 = largest e2m1 magnitude); scales: float [T]. */
    PERQ_FMT_FP4_TOKEN = 3,
    /* The same with the step as that paragraph prints it, s = max|y| / (2^(q-1) - 1) = max|y| / 7:
     * values above 6.5 steps, the row maximum among them, saturate to the largest code. */
    PERQ_FMT_FP4_TOKEN_AMAX7 = 4
} perq_fmt_t;

/* Which rotation kernel runs.  AUTO picks the fastest one that covers the shape (block sizes that
 * are not powers of two, and powers of two above 4096 on rows of 8192, 16384 or 32768, have a
 * matrix-core kernel of their own that only AUTO selects); the explicit values exist so that the
 * two general kernels can be compared with each other and each checked alone. */
typedef enum {
    PERQ_ALGO_AUTO = 0,
    PERQ_ALGO_BUTTERFLY = 1,  /* register / cross-lane / LDS radix-2 butterflies; every shape with a
                                 power-of-two b */
    PERQ_ALGO_MFMA = 2        /* X * H on the matrix cores for the low index bits (b <= 4096, d a
                                 multiple of 512); UNSUPPORTED for shapes it does not cover */
} perq_algo_t;

/* Largest row width the kernels accept (elements). */
#define PERQ_MAX_D 32768

const char* perq_status_string(perq_status_t status);

/*
 * Column statistic of Algorithm 1 (its sort key): out_mean[i] = (1/M) * sum_k |x[k, i]|.
 *
 *   x_bf16     device, bf16 [M, ldx], ldx >= d, ldx % 8 == 0 and base 16-byte aligned
 *   out_mean   device, float [d]
 *   workspace  device, at least perq_colabs_mean_workspace_bytes(M, d) bytes, 16-byte aligned
 *
 * Two deterministic passes (row-slice partial sums in fp32, then a fixed-order reduction);
 * the result does not depend on scheduling.  M == 0 is INVALID_ARG (the mean is undefined).
 * Accuracy: a partial sum adds at most r - 1 non-negative fp32 terms, r = rows per slice =
 * max(8, ceil(M / floor(512 / ceil(d / 2048)))), and the second pass works in double, so
 * |out_mean[i] - a_i| < (r + 1) 2^-24 a_i  (r <= 32 for M <= 4096: below 2.0e-6 relative).
 */
size_t perq_colabs_mean_workspace_bytes(int64_t M, int32_t d);
perq_status_t perq_colabs_mean(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx,
                               float* out_mean, void* workspace, size_t workspace_bytes,
                               void* hip_stream);

/*
 * perq_colabs_mean for callers that cannot allocate device memory or hand any over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same result
 * bit for bit; the partial sums live in a 4 MiB array that is part of the library's code object
 * (one copy per device, held until the process ends) instead of a caller's workspace.  The call
 * itself allocates and frees nothing.  The very first call on a device looks up the array's
 * address there; make that call outside a capture.
 *   Limit: perq_colabs_mean_workspace_bytes(M, d) <= 4 MiB, which holds for every M when
 *   d <= 1048576; beyond it PERQ_ERR_UNSUPPORTED.  Other arguments and errors as perq_colabs_mean.
 *   All calls on one device share the array: two calls that overlap there (different streams, or
 *   graph replays side by side) race and give undefined means; calls on one stream are safe.
 *   Nothing needs clearing between calls (the first pass overwrites every partial the second reads).
 */
perq_status_t perq_colabs_mean_static(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx,
                                      float* out_mean, void* hip_stream);

/*
 * max_k |x[k, i]| per channel, the statistic of the "absmax" and ZigZag permutations compared in
 * Appendix C ("Permutations").  Arguments, workspace size and errors as perq_colabs_mean; exact.
 */
perq_status_t perq_colabs_absmax(const uint16_t* x_bf16, int64_t M, int32_t d, int64_t ldx,
                                 float* out_max, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/*
 * Algorithm 1 (mass diffusion), host side, on the sufficient statistic a = colabs_mean.
 *
 *   colabs_mean  host, float [d], finite and >= 0
 *   perm_out     host, int32 [d]; perm_out[j*b + k] = k-th channel placed in block j
 *
 * Channels are visited by descending a (ties: lower channel first); each goes to the not-yet-
 * full block of least accumulated mass (ties: lowest block).  Masses accumulate in double.
 * Any b >= 1 dividing d is accepted here (the rotation's b >= 16 limit does not apply).
 */
perq_status_t perq_massdiff_perm(const float* colabs_mean, int32_t d, int32_t b, int32_t* perm_out);

/*
 * The other calibrated permutations of Appendix C ("Permutations"), host side, same output
 * convention as perq_massdiff_perm.  stat: host, float [d], finite and >= 0.
 *   perq_perm_sorted  "absmax": channels in descending order of stat (ties: lower channel first).
 *   perq_perm_zigzag  the paper only names the strategy; taken: rank r of that order goes to block
 *                     r mod n on even rounds floor(r/n) and to block n-1-(r mod n) on odd rounds
 *                     (n = d/b), each block in arrival order.
 *   perq_perm_random  the ablation's random permutation, reproducible: Fisher-Yates from the top down
 *                     (i = d-1 .. 1, swap positions i and floor(u (i+1) / 2^64)), u the successive
 *                     outputs of SplitMix64 (Steele, Lea, Flood 2014) started at `seed`.  No stat.
 */
perq_status_t perq_perm_sorted(const float* stat, int32_t d, int32_t* perm_out);
perq_status_t perq_perm_zigzag(const float* stat, int32_t d, int32_t b, int32_t* perm_out);
perq_status_t perq_perm_random(int32_t d, uint64_t seed, int32_t* perm_out);

/*
 * The 4t-dimensional base matrix of the rotation for a block size that is not a power of two
 * (Appendix A.1, "An Optimized Non-Power-of-2 Hadamard Rotation"): b = 2^k' * m, m = 4t, t odd, and
 * R = (H_{2^k'} (x) H_m) / sqrt(b), H_{2^k'} Sylvester's matrix, position a*m + r of a block
 * belonging to row a of the first factor and row r of the second.  The appendix prints no base
 * matrix; the library takes Paley's constructions over a prime field, Q[i][j] = chi(i - j):
 *   m - 1 prime, = 3 mod 4:    H_m = I + [[0, 1^T], [-1, Q]]                          (m = 12)
 *   else m/2 - 1 prime, = 1 mod 4:  [[0, 1^T], [1, Q]] with 0 -> [[1,-1],[-1,-1]] and
 *                                   e = +-1 -> e [[1,1],[1,-1]]                       (m = 28, 76)
 *   out   host, int8 [m][m], entries +-1; a row vector x is rotated as x H_m
 * INVALID_ARG when m is not 4t with t odd and above 1, or neither construction exists for it.  Needed offline to rotate the weights that
 * meet the activations (W~ = R~^T P^T W).
 */
perq_status_t perq_hadamard_base(int32_t m, int8_t* out);

/* OK iff perm (host, int32 [d]) is a bijection on [0, d); INVALID_ARG otherwise. */
perq_status_t perq_perm_validate(const int32_t* perm_host, int32_t d);

/*
 * Host.  perm arranged for the fused kernel's operand gather.  With a permutation the kernel
 * fetches every operand element with a 2-byte LDS read of its own, and on arbitrary channel
 * orders the lanes of one read instruction meet in the same LDS banks.  Algorithm 1 decides which
 * channels share a block -- that fixes the block masses and with them the bound of Proposition 2
 * and Corollary 3.3 -- while those bounds do not depend on the order inside a block or on the
 * place of a block in the row, and P is merged into the neighbouring weights whatever it is
 * (Section 4, remark on merging permutations).  perq_perm_arrange keeps the channel set of every block of b positions, deals
 * the blocks to the kernel's 4096-wide tiles so that every tile's channels spread evenly over the
 * banks, and orders every block so that the lanes of a read instruction meet different banks.
 * The result is a different permutation with the same blocks: whatever is merged offline must be
 * merged with perm_out.  Shapes the arrangement does not apply to (d < 4096, d % 512 != 0,
 * b > 4096, b not a power of two) are copied unchanged.
 * The typical error does depend on the order in one respect: Algorithm 1 fills a block heaviest channel
 * first, so the outlier channels of a block meet the first columns of H_b, whose sums take few
 * distinct values.  On blocks that hold several outliers (b >= 512) the per-token INT4 error of the
 * synthetic workloads is 2-15 % lower in that order than in any other order of the same sets
 * (MXFP4, and any format at b <= 256: no difference).  `head` positions at the start of every
 * block therefore keep the channels they were given: head < 0 means 64 for b >= 512 and 0 below,
 * head = 0 moves everything.  If the result would cost more passes (perq_perm_gather_cost) than
 * perm itself, perm is returned.
 *   perm, perm_out  host, int32 [d]; perm must be a bijection on [0,d); may be the same array
 *   head            -1, or 0 .. b
 * perq_perm_gather_cost reports what the arrangement is about: `reads` = read instructions per
 * half-wave and row, `passes` = the sum over them of the largest number of lanes that meet in one
 * bank on different words (passes == reads: no conflicts).  PERQ_ERR_UNSUPPORTED for the shapes
 * listed above.
 */
perq_status_t perq_perm_arrange(const int32_t* perm, int32_t d, int32_t b, int32_t head, int32_t* perm_out);
perq_status_t perq_perm_gather_cost(const int32_t* perm, int32_t d, int32_t b, int64_t* passes, int64_t* reads);

/*
 * The fused online path: gather through perm, rotate every b-block, quantize, pack.
 *
 *   x_bf16   device, bf16 [T, ldx]; ldx >= d; base 16-byte aligned and ldx % 8 == 0
 *   perm     device, int32 [d], or NULL for P = I
 *   b        16 <= b <= d, b divides d; a power of two, or 2^k' * 4t with 4t = 28 (d = 3584, 7168,
 *            14336, 28672), 4t = 12 (d = 3072, 6144, 12288) or 4t = 76 (d = 2432, 4864, 9728); see
 *            perq_hadamard_base.  Other widths for these bases, and other bases the library can
 *            build, are UNSUPPORTED; a b for which it knows no Hadamard matrix is INVALID_ARG
 *   codes    device, uint8 [T, d/2]; element 2k in the low nibble of byte k, 2k+1 in the high
 *   scales   INT4:  device float [T], s_t = ||y_t||_inf / 7 (0 for an all-zero row)
 *            MXFP4: device uint8 [T, d/32], biased exponent E, scale = 2^(E-127),
 *                   E - 127 = floor(log2 ||group||_inf) - 2, clamped to [0,254], 0 for a zero group
 *            INT4_ASYM_TOKEN: device float [T][2] = (step, zero point); FP4_TOKEN(_AMAX7): device float [T]
 *                   (see perq_fmt_t)
 *   d % 32 == 0 is required for both formats; T == 0 is OK and does nothing.
 *
 * Rounding is to nearest, ties to even; MXFP4 saturates at +-6 and always writes zero as +0.
 */
perq_status_t perq_permute_rotate_quant(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                        const int32_t* perm, int32_t b, perq_fmt_t fmt,
                                        uint8_t* codes, void* scales, void* hip_stream);

/*
 * A permutation prepared for the main kernel (host, once per layer), and the fused call that uses it.
 * Two things are worked out ahead of the launches; P itself is untouched and so is every output bit.
 *   Operand offsets.  With a permutation the kernel fetches every operand element with a 2-byte LDS
 * read at an address that depends on perm, the lane and the kernel's operand layout.  The plain call
 * turns perm into these addresses at the start of every launch (about 5 us of a short launch); the
 * prepared form holds them as 16-bit offsets in the order the lanes need them, for both of the
 * kernel's operand layouts (b <= 512 and b >= 1024), so a lane fetches its 64 offsets with eight
 * 16-byte loads issued ahead of its first row loads.
 *   Placement (rows wider than 8192).  Where a row's 16-byte pieces lie in LDS decides how many of the
 * 32 lanes of a read meet in one bank.  The kernel's fixed layout serves P = I and regular patterns; on
 * an arbitrary permutation a read takes 3.2 - 3.5 passes.  perq_perm_prepare picks, for the permutation
 * at hand, the group of four banks every piece of eight channels lands in (the loads that stage the row
 * stay as coalesced as they are: pieces move only inside their 128-byte line of the row), which brings
 * a read to about 2.3 passes.  Rows of one or two tiles keep the fixed layout: the lookup that would
 * have to come before a workgroup's first row loads costs them more than the reads gain.
 * Once per layer; 6 ms for d = 4096, 25 ms for d = 14336 on one host core.
 *   perq_perm_prepared_bytes   size of the prepared form for rows of d channels: d int32 (per position,
 *                              the place of its channel in the staged row: slot * 8 + channel % 8),
 *                              d / 8 uint16 (the piece of the row in every slot), then two tables
 *                              (b <= 512, b >= 1024) of ceil(d / 4096) * 4096 uint16 each: per tile of
 *                              4096 positions, operand fragment (8), lane (64) and element (8) the byte
 *                              offset of that operand in the staged row (fixed layout for d <= 8192,
 *                              else the placement; 0xFFFF past the end of the row); 0 if d is not a
 *                              positive multiple of 8
 *   perq_perm_prepare          perm: host, int32 [d], a bijection; b: the block size the fused call
 *                              will be made with (the placement is chosen for the read pattern of
 *                              b <= 512 or of b >= 1024; the output is correct with either);
 *                              prepared: host, out, perq_perm_prepared_bytes(d);
 *                              passes_before / passes_after / reads (each may be NULL): the sum over
 *                              the read instructions of a row of the largest number of lanes per
 *                              bank, with the fixed layout and with the chosen placement, and their
 *                              number.  Never worse than the fixed layout.  UNSUPPORTED for shapes
 *                              whose kernel has no such gather (d < 4096, d % 512 != 0, b > 4096 or
 *                              not a power of two).
 *   perq_perm_prepared_validate  OK iff `prepared` (host) is what some placement gives for `perm`: every
 *                              piece inside its line of 8, every slot taken once, every position's
 *                              place that of its channel, every operand offset the one that follows
 *   perq_permute_rotate_quant_prepared   perq_permute_rotate_quant with the prepared form (device,
 *                              16-byte aligned, a copy of all perq_perm_prepared_bytes(d) bytes that
 *                              perq_perm_prepare wrote for this perm and d; or NULL: the plain call).
 *                              perm is still passed: calls that do not run on the main kernel with a
 *                              permutation use it and ignore `prepared`.
 *                              `prepared` is not checked on the device.  Its entries address LDS only
 *                              (an offset past the staged rows reads zero or another row's data, never
 *                              outside the workgroup's memory) and pieces of the row (clipped to the
 *                              row), so a form that does not belong to perm gives undefined output
 *                              values and nothing else; a buffer shorter than
 *                              perq_perm_prepared_bytes(d) is read past its end.  Any valid form gives
 *                              the outputs of the plain call, bit for bit.
 */
size_t perq_perm_prepared_bytes(int32_t d);
perq_status_t perq_perm_prepare(const int32_t* perm, int32_t d, int32_t b, void* prepared,
                                int64_t* passes_before, int64_t* passes_after, int64_t* reads);
perq_status_t perq_perm_prepared_validate(const void* prepared, const int32_t* perm, int32_t d);
perq_status_t perq_permute_rotate_quant_prepared(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                                 const int32_t* perm, const void* prepared, int32_t b,
                                                 perq_fmt_t fmt, uint8_t* codes, void* scales,
                                                 void* hip_stream);

/* Same as perq_permute_rotate_quant with the rotation kernel chosen by the caller. */
perq_status_t perq_permute_rotate_quant_algo(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                             const int32_t* perm, int32_t b, perq_fmt_t fmt,
                                             perq_algo_t algo, uint8_t* codes, void* scales,
                                             void* hip_stream);

/*
 * Test entry: the same gather + rotation device code as perq_permute_rotate_quant(_algo),
 * writing the pre-quantization values y = (XP R~)[T, d] as float (normalised by 1/sqrt(b)).
 *   y   device, float [T, d], 16-byte aligned
 */
perq_status_t perq_permute_rotate_f32(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                      const int32_t* perm, int32_t b, perq_algo_t algo,
                                      float* y, void* hip_stream);

/*
 * Per-token quantities of Section 3 for a given permutation and block size (device):
 *   out[t] = ( ||x_t||_inf,  ||x_t||_1,  max_j ||(x_t P)_{j}||_1,  ||x_t P R~||_inf )     float [T][4]
 * so that delta = out[1] / (d out[0]) (Proposition 1), the bound of Proposition 2 and Z(b; xP) of
 * Corollary 3.3 are out[2] / sqrt(b), and the outlier suppression ratio is out[3] / out[0].
 * Arguments and errors as perq_permute_rotate_f32; out 16-byte aligned.  fp32 sums in a fixed order.
 */
perq_status_t perq_block_diagnostics(const uint16_t* x_bf16, int64_t T, int32_t d, int64_t ldx,
                                     const int32_t* perm, int32_t b, float* out, void* hip_stream);

/*
 * Per-token quantization error of an output of the fused path (Section 3: the worst-case l2 error of
 * a q-bit quantizer with step ||y||_inf / (2^(q-1) - 1) is sqrt(d) / (2^q - 2) ||y||_inf, the reason
 * outliers are suppressed at all):
 *   out[t] = ( ||y_t - Q(y_t)||_2,  ||y_t||_2,  ||y_t||_inf )                          float [T][3]
 *   y       device, float [T, d], the output of perq_permute_rotate_f32, 8-byte aligned
 *   codes   device, uint8 [T, d/2], and
 *   scales  device, as perq_permute_rotate_quant wrote them for the same input, perm, b and fmt
 * Q(y) is the value the codes stand for: step * code (INT4), step * (code + zero point) (asymmetric
 * INT4), step * e2m1 value (FP4 per token), 2^(E-127) * e2m1 value (MXFP4).  d % 32 == 0.  fp32 sums in
 * a fixed order.  T == 0 does nothing.
 */
perq_status_t perq_quant_error(const float* y, int64_t T, int32_t d, const uint8_t* codes,
                               const void* scales, perq_fmt_t fmt, float* out, void* hip_stream);

/*
 * Reference consumer of the codes (Remark "Merging Permutations", Section 4): with P and the block
 * rotation merged into the weights, W~ = R~^T P^T W, the product of the two quantized operands
 * stands for X W.  Both operands are PERQ_FMT_INT4_SYM_TOKEN outputs of
 * perq_permute_rotate_quant: the activations [T, d], and the weights as the rows of W^T [N, d] run
 * through the same perm and b (one step per output channel).
 *
 *   out[t, n] = a_scales[t] * w_scales[n] * sum_i a_code[t, i] * w_code[n, i]
 *
 *   a_codes  device, uint8 [T, d/2], 16-byte aligned;   a_scales  device, float [T]
 *   w_codes  device, uint8 [N, d/2], 16-byte aligned;   w_scales  device, float [N]
 *   out      device, float [T, ldo], ldo >= N
 * The integer sums are exact; the two multiplications are fp32, left to right.  A plain integer
 * kernel for checking the layout end to end, not a tuned GEMM.  T == 0 or N == 0 does nothing.
 */
perq_status_t perq_w4a4_gemm_ref(const uint8_t* a_codes, const float* a_scales, int64_t T,
                                 const uint8_t* w_codes, const float* w_scales, int32_t N, int32_t d,
                                 float* out, int64_t ldo, void* hip_stream);

/*
 * The same for PERQ_FMT_MXFP4 operands (Appendix B, Eq. 5): both are outputs of
 * perq_permute_rotate_quant, e2m1 codes with one e8m0 byte per 32.
 *
 *   out[t, n] = sum over 32-groups g of 2^(Ea[t,g] - 127) 2^(Ew[n,g] - 127) sum_{i in g} a[t,i] w[n,i]
 *
 *   a_codes  device, uint8 [T, d/2], 16-byte aligned;   a_scales  device, uint8 [T, d/32]
 *   w_codes  device, uint8 [N, d/2], 16-byte aligned;   w_scales  device, uint8 [N, d/32]
 *   out      device, float [T, ldo], ldo >= N
 * Runs on gfx950's scaled matrix instruction (v_mfma_scale_f32_32x32x64_f8f6f4, fp4 x fp4), which
 * takes a 32-group of packed codes and its scale byte exactly as the fused path writes them: the
 * products are exact, the sums are fp32 in the unit's own order.  A checker of the layout, not a
 * tuned GEMM.  d % 32 == 0; T == 0 or N == 0 does nothing.
 */
perq_status_t perq_w4a4_mxfp4_gemm_ref(const uint8_t* a_codes, const uint8_t* a_scales, int64_t T,
                                       const uint8_t* w_codes, const uint8_t* w_scales, int32_t N, int32_t d,
                                       float* out, int64_t ldo, void* hip_stream);

/*
 * The run-time row schedule of the main kernel (see "Conventions" above).
 *   perq_schedule_set    the counter set launches on `hip_stream` draw from, 0 .. 63 (assigned at
 *                        the first call for that stream, by this function or by a launch), or -1
 *                        when such launches take the fixed split: the stream is capturing, or 64
 *                        other streams of the current device came first.
 *   perq_reset_schedule  enqueues a small kernel on `hip_stream` that puts every counter of the
 *                        current device back to zero.  Never needed after launches that ran to
 *                        their end; for a process that goes on after a kernel of the library was
 *                        cut short.  Must not overlap a launch of the fused path on another stream.
 *   perq_schedule_selftest  host only: a model of the schedule on the kernel's own queue
 *                        arithmetic -- n_blocks workgroups of workers_per_block workers each draw
 *                        their units in a seeded random interleaving, `launches` times on the same
 *                        counters.  OK iff every unit was taken exactly once, every queue handed out
 *                        units + workers tickets and every counter ended at zero; UNSUPPORTED for a
 *                        shape that would not use the queues (n_blocks % 256 != 0 or fewer than two
 *                        units per worker); INTERNAL on a violation.
 */
int32_t perq_schedule_set(void* hip_stream);
perq_status_t perq_reset_schedule(void* hip_stream);
perq_status_t perq_schedule_selftest(int64_t n_units, int32_t n_blocks, int32_t workers_per_block,
                                     uint64_t seed, int32_t launches);

#ifdef __cplusplus
}
#endif
#endif /* PERQ_H */
