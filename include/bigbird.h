/*
 * bigbird.h -- C ABI of the MI355X (gfx950) BigBird block-sparse attention library.
 *
 * The library evaluates, per head, the generalised attention of Sec. 2, eq. (AT)
 * with sigma = softmax on the BigBird graph in its blocked form (App. D): with
 * block length b, query block j attends the g global key blocks, the w window
 * key blocks j-(w-1)/2 .. j+(w-1)/2 and the r random key blocks listed in
 * rand_idx[h][j][:]; global query blocks attend every key block (Sec. 2, ITC:
 * A(i,:) = 1 and A(:,i) = 1 for i in G).  The residual "x_i +" and the sum over
 * heads in eq. (AT) belong to the caller: outputs are per head.
 *
 * Conventions that hold for every entry point
 *   - plain C linkage, no exceptions cross the boundary, the int return value
 *     (a BB_* status) is the only error channel, no global state;
 *   - "device" pointers are HIP device memory on the current device, "host"
 *     pointers ordinary host memory; the caller owns every buffer, the library
 *     never allocates or frees device memory and keeps no pointer after return;
 *   - tensors are contiguous row-major; Q, K, V, O, dO are [B][H][n][d] in the
 *     storage type named by `dtype`; LSE and all gradients are fp32;
 *   - device work is enqueued on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and the call returns without synchronising;
 *   - outputs are fully overwritten, never accumulated into;
 *   - everything checkable on the host is checked before the first launch, and a
 *     failed check launches nothing.  The device copy of rand_idx is trusted by
 *     the attention calls: check the table with bigbird_validate_rand_idx first.
 *   - supported shapes: d == 64, b == 64, n a positive multiple of b, w odd >= 1,
 *     0 <= g <= n/b, r >= 0, scale finite and > 0 (eq. (AT) carries no scale; any
 *     positive one can be folded into Q_h).  Anything else is BB_ERR_SHAPE or
 *     BB_ERR_UNSUPPORTED, never a silent wrong answer.  B == 0 or H == 0 is a
 *     valid empty problem (BB_OK, nothing launched).
 *   - overlapping components form a set union (A is 0/1, Sec. 2): a key block
 *     that is global and in the window is attended once.
 */
#ifndef BIGBIRD_H_
#define BIGBIRD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  BB_OK = 0,
  BB_ERR_NULL = -1,        /* a required pointer is NULL */
  BB_ERR_SHAPE = -2,       /* sizes violate the conventions above */
  BB_ERR_PATTERN = -3,     /* rand_idx invalid, or too few candidate blocks for r */
  BB_ERR_DTYPE = -4,       /* dtype is not BB_F32 / BB_BF16 */
  BB_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than bigbird_attn_workspace_bytes */
  BB_ERR_UNSUPPORTED = -6, /* legal in the paper's terms but not built (d != 64, b != 64, ...) */
  BB_ERR_LAUNCH = -7       /* the HIP runtime refused a launch */
};

enum { BB_F32 = 0, BB_BF16 = 1 };

/* Placement of the g global blocks (Sec. 2 says "a subset G"; App. D says "the
 * first g blocks").  FIRST_LAST: ceil(g/2) leading and floor(g/2) trailing
 * blocks; LEADING: blocks 0 .. g-1. */
enum { BB_GLOBAL_FIRST_LAST = 0, BB_GLOBAL_LEADING = 1 };

/* Option flag, OR-ed into the global_mode argument of the attention calls and of
 * bigbird_count_block_pairs (the paper has no padding; this is a reading of the mask).  With
 * it the key-padding mask is also read as a query mask, block by block: a query block in
 * which every position is padded is not computed -- its rows get O = 0, LSE = -inf, send
 * no gradient to K and V and receive dQ = 0 -- the way a caller that never reads padded rows
 * wants them.  Query blocks with at least one valid position are computed in full, as
 * without the flag.  Ignored when there is no mask.  Give the backward call the flag the
 * forward call had. */
enum { BB_SKIP_PADDED_QUERY_BLOCKS = 0x100 };

/* Human-readable name of a status code.  Never NULL. */
const char* bigbird_status_string(int status);

/*
 * Random component of the pattern (App. D item 1: every query block attends
 * exactly r random key blocks).  Host only, integers only, deterministic.
 * Fills rand_idx_host[H][n/b][r] (int32): for each head h and non-global query
 * block j, r distinct key blocks drawn uniformly without replacement from the
 * blocks outside window(j) and outside G, stored ascending; rows of global query
 * blocks are -1.  The generator is counter based: a 64-bit SplitMix finaliser
 * keyed by (seed, h, j, draw), rejection sampling for bounded integers, partial
 * Fisher-Yates over the ascending candidate list.
 * Errors: BB_ERR_NULL, BB_ERR_SHAPE, BB_ERR_PATTERN (a row has fewer than r
 * candidates).
 */
int bigbird_make_rand_idx(int32_t* rand_idx_host, int H, int n, int b, int g, int w, int r,
                          uint64_t seed, int global_mode);

/*
 * Host check of a table laid out as above: every non-global row must hold r
 * distinct blocks in [0, n/b) outside window(j) and G.  Rows of global query
 * blocks are ignored.  BB_OK or BB_ERR_PATTERN (BB_ERR_NULL / BB_ERR_SHAPE for
 * bad arguments).
 */
int bigbird_validate_rand_idx(const int32_t* rand_idx_host, int H, int n, int b, int g, int w,
                              int r, int global_mode);

/*
 * Number of (query block, key block) pairs of the pattern summed over batch and
 * heads: the unit of useful work (4 b^2 d flop forward per pair, App. D cost
 * O(n (g+w+r) b d)).  key_mask_host is NULL or [B][n] bytes (non-zero = valid
 * key); with a mask, pairs whose key block holds no valid key are not counted.
 * Host only.  Returns the count, or a negative BB_* status.
 */
int64_t bigbird_count_block_pairs(const int32_t* rand_idx_host, const uint8_t* key_mask_host,
                                  int B, int H, int n, int b, int g, int w, int r,
                                  int global_mode);

/*
 * Bytes of device scratch the attention calls need for these sizes (partial
 * results of rows / columns that are split over several workgroups; with
 * need_bwd != 0 also the backward's row sums and partial gradients).  Returns 0
 * for invalid sizes.  The workspace must be 256-byte aligned; its contents need
 * not be initialised and are undefined afterwards.
 */
size_t bigbird_attn_workspace_bytes(int B, int H, int n, int d, int b, int g, int w, int r,
                                    int need_bwd);

/*
 * Forward pass, eq. (AT) per head on the blocked BigBird graph (App. D):
 *   S = scale * Q K^T restricted to the pattern and to valid keys,
 *   LSE_i = ln sum_k exp(S_ik),  O_i = sum_k exp(S_ik - LSE_i) V_k.
 * Q, K, V   device [B][H][n][d], dtype BB_BF16 (bf16 storage, fp32 accumulation,
 *           probabilities rounded to bf16 before the P V product) or BB_F32;
 * O         device [B][H][n][d], same dtype; LSE device [B][H][n] fp32
 *           (natural log, includes scale);
 * rand_idx  device [H][n/b][r] int32 (may be NULL when r == 0); entries < 0 are
 *           ignored; duplicates of window / global / earlier entries are dropped;
 * key_padding_mask  NULL, or device [B][n] bytes, non-zero = valid key.  Padded
 *           keys are removed for every query (global rows too); padded queries are
 *           still computed; a row with no valid key gives O = 0, LSE = -inf.
 * Pointers must be 16-byte aligned.
 */
int bigbird_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                     const int32_t* rand_idx, const uint8_t* key_padding_mask,
                     int B, int H, int n, int d, int b, int g, int w, int r,
                     float scale, int dtype, int global_mode,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * bigbird_attn_fwd for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, checks, kernels and results as
 * bigbird_attn_fwd, without the workspace: the scratch memory is a static device
 * array of BIGBIRD_STATIC_SCRATCH_BYTES inside the library (one per GPU, held
 * until the process ends).  The call allocates and frees nothing.  Sizes for which
 * bigbird_attn_workspace_bytes(..., need_bwd = 0) exceeds that limit are refused
 * with BB_ERR_WORKSPACE and a message on stderr.  The device the arrays live on is
 * the current device of the calling thread (hip_stream must belong to it);
 * BB_ERR_LAUNCH if the array's address cannot be obtained.  All calls on one GPU
 * share its array, which keeps the previous call's partial results: nothing in it
 * has to be cleared between calls, but calls that overlap in time on one GPU
 * (different streams, different threads) race and give undefined results.
 */
#define BIGBIRD_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int bigbird_attn_fwd_static(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            const int32_t* rand_idx, const uint8_t* key_padding_mask,
                            int B, int H, int n, int d, int b, int g, int w, int r,
                            float scale, int dtype, int global_mode, void* hip_stream);

/*
 * Backward pass (the paper gives none: calculus on eq. (AT)).  With P the row
 * softmax recomputed from Q, K and LSE:
 *   dV = P^T dO;  dP = dO V^T;  D_i = sum_c dO_ic O_ic;  dS = P o (dP - D);
 *   dQ = scale dS K;  dK = scale dS^T Q.
 * O, LSE are the forward's outputs for the same inputs; dO has the layout and
 * dtype of O; dQ, dK, dV are device [B][H][n][d] fp32, fully overwritten.  The
 * reduction over the random-block scatter is atomic free (fixed summation order,
 * bit-reproducible).  Gradients of padded keys are exactly 0.
 * The workspace must have been sized with need_bwd != 0.
 * dtype BB_BF16 (the tuned path) or BB_F32 (fp32 end to end, plain kernels: a correctness
 * configuration).  BB_ERR_UNSUPPORTED for n / b > 256.
 */
int bigbird_attn_bwd(const void* Q, const void* K, const void* V, const void* O,
                     const float* LSE, const void* dO, float* dQ, float* dK, float* dV,
                     const int32_t* rand_idx, const uint8_t* key_padding_mask,
                     int B, int H, int n, int d, int b, int g, int w, int r,
                     float scale, int dtype, int global_mode,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Attention dropout (the paper names only the rate: "attention dropout 0.1", App. E.1
 * hyper-parameter table).  Reading: after the row softmax of eq. (AT) every attended
 * probability P_ij is kept with probability 1 - p and the kept ones are scaled by
 * 1 / (1 - p), independently per (batch, head, query i, key j); LSE stays that of the
 * undropped softmax:
 *   O_i = sum_j M_ij / (1 - p) P_ij V_j.
 * The keep mask M is a function of (seed, bh = batch * H + head, i, j) alone, so that the
 * forward and the backward of one step, called with the same p_drop and seed, see the same
 * mask.  Counter-based generator on 32-bit integers (arithmetic modulo 2^32):
 *   mix(x):  x ^= x >> 16; x *= 0x7feb352d; x ^= x >> 15; x *= 0x846ca68b; x ^= x >> 16
 *   rk(i)   = mix(seed_lo ^ mix(seed_hi ^ (bh * n + i)))
 *   w(i, j) = mix(rk(i) ^ ((j >> 1) * 0x9E3779B9))
 *   u(i, j) = bits 0..14 of w for even j, bits 16..30 for odd j
 *   M_ij    = [ u(i, j) >= T ],  T = round(p_drop * 32768)
 * so the rate realised is T / 32768 (0.100006 for 0.1) and the scale 32768 / (32768 - T).
 * p_drop must lie in [0, 1) with T < 32768, else BB_ERR_SHAPE (checked before anything
 * else); p_drop == 0 is the plain call, bit for bit.  Use a new seed for every step and layer.
 *
 * bigbird_attn_fwd_dropout: arguments, checks and outputs of bigbird_attn_fwd, plus p_drop and
 * seed.  The bf16 path applies the mask on its per-item path (the one that also serves
 * blocks with padded keys inside), not in the pipelined one: expect about half the
 * throughput of the plain call.
 */
int bigbird_attn_fwd_dropout(const void* Q, const void* K, const void* V, void* O, float* LSE,
                             const int32_t* rand_idx, const uint8_t* key_padding_mask,
                             int B, int H, int n, int d, int b, int g, int w, int r,
                             float scale, int dtype, int global_mode,
                             float p_drop, uint64_t seed,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of bigbird_attn_fwd_dropout (same p_drop and seed; O and LSE from that call), mask
 * held fixed:  dV = (M o P / (1-p))^T dO;  dP = M / (1-p) o (dO V^T);  D_i = sum_c dO_ic O_ic;
 * dS = P o (dP - D);  dQ = scale dS K;  dK = scale dS^T Q.  Otherwise as bigbird_attn_bwd.
 */
int bigbird_attn_bwd_dropout(const void* Q, const void* K, const void* V, const void* O,
                             const float* LSE, const void* dO, float* dQ, float* dK, float* dV,
                             const int32_t* rand_idx, const uint8_t* key_padding_mask,
                             int B, int H, int n, int d, int b, int g, int w, int r,
                             float scale, int dtype, int global_mode,
                             float p_drop, uint64_t seed,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The keep mask itself, on the host (integers only; what the kernels compute element by
 * element): rows row0 .. row0 + nrows - 1 of slice bh, keep_host[nrows][n] bytes (1 = kept).
 * scale_out (may be NULL) receives 32768 / (32768 - T).  BB_ERR_NULL, BB_ERR_SHAPE.
 */
int bigbird_dropout_keep_mask(uint8_t* keep_host, float* scale_out, float p_drop, uint64_t seed,
                              int bh, int n, int row0, int nrows);

#ifdef __cplusplus
}
#endif
#endif /* BIGBIRD_H_ */
