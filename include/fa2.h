/*
 * libfa2 -- fused scaled dot-product attention forward pass for AMD MI355X (gfx950 / CDNA4).
 *
 * The operation is the one stated in Section 2 of "A Case Study in CUDA Kernel Fusion:
 * Implementing FlashAttention-2 on NVIDIA Hopper Architecture using the CUTLASS Library"
 * (arXiv 2312.11918):
 *
 *      O = softmax(scale * Q K^T) V        independently for every batch entry and head,
 *
 * computed as in its Algorithm 2 (FlashAttention-2 forward): for each tile of query rows the
 * kernel streams tiles of K and V, forms S = Q K^T on the matrix cores, keeps a running row
 * maximum and row sum (online softmax), accumulates O = P V on the matrix cores and divides by
 * the row sum at the end.  S and P live in registers only and never reach device memory.
 *
 * Besides O the library returns the row-wise log-sum-exp of the scaled logits,
 *      LSE[b,h,i] = ln sum_j exp(scale * q_i . k_j),
 * which Algorithm 2 holds implicitly as (rowmax, rowsum) and which callers need to merge
 * attention computed over disjoint key ranges.
 *
 * Plain C ABI: pointers and sizes only.  Every data pointer is a DEVICE pointer owned by the caller.
 */
#ifndef FA2_H_
#define FA2_H_

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of Q, K, V and O. */
enum { FA2_FP16 = 0, /* IEEE binary16 */
       FA2_BF16 = 1  /* bfloat16      */ };

/* Return codes. */
enum {
  FA2_OK = 0,
  FA2_ERR_INVALID_ARG = -1, /* NULL Q/K/V/O; B, H, N or d <= 0; scale not finite or <= 0;
                               a pointer not 16-byte aligned (LSE: 4-byte); an unknown
                               variant or mask                                        */
  FA2_ERR_UNSUPPORTED = -2, /* d not in {64, 128, 256}; unknown dtype; a problem too large
                               for 32-bit tile counts and offsets; a tile shape or mask
                               that cannot run the given sizes (see each entry point)  */
  FA2_ERR_LAUNCH = -3       /* the HIP runtime refused the launch                     */
};

/*
 * fa2_fwd -- attention forward pass (Section 2 formula, Algorithm 2 schedule), non-causal,
 * no mask, no dropout, self-attention shape (as many keys as queries).
 *
 *  Q, K, V  in   device, [B][N][H][d] contiguous, element (b,n,h,k) at ((b*N+n)*H+h)*d+k
 *                (the paper's (batch, seqlen, heads, headdim) order), 16-bit elements of `dtype`.
 *  O        out  device, same shape, layout and element type as Q.  Rounded once, from the fp32
 *                accumulator, to nearest-even.
 *  LSE      out  device, [B][H][N] contiguous fp32, natural logarithm; may be NULL (not written).
 *  B,H,N,d       batch, heads, sequence length, head dimension.  d must be 64, 128 or 256 (the head
 *                dimensions of the paper's benchmarks, Section 7); N is any length >= 1 (a length
 *                that is not a multiple of 128 runs a kernel variant that masks the partial tiles).
 *  scale         multiplies Q K^T before the softmax; callers pass 1/sqrt(d).  Must be finite
 *                and > 0 (the kernel takes the row maximum before scaling).
 *  dtype         FA2_FP16 or FA2_BF16.  Products are accumulated in fp32; P is rounded to `dtype`
 *                (nearest-even) before the second matrix product, the row sum is taken in fp32
 *                from the unrounded P.
 *  stream        a hipStream_t passed as void*; NULL is the default stream.
 *
 * The call only enqueues one kernel on `stream` and returns; it allocates nothing, keeps no state
 * and never synchronises.  Buffers must stay valid until the stream has run the kernel.  O and LSE
 * must not overlap Q, K or V.  On any error nothing is launched and the outputs are untouched.
 * Inputs holding NaN or infinities give unspecified outputs.  Safe to call from several threads.
 * The launch uses the device that is current on the calling thread; all pointers must belong to it.
 */
int fa2_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N, int d,
            float scale, int dtype, void* stream);

/* Tile shapes (the counterpart of the paper's QBLK x KBLK choice, Section 7 and Table 1). */
enum {
  FA2_VARIANT_AUTO = 0,   /* pick by problem shape (what fa2_fwd does)                                  */
  FA2_VARIANT_NARROW = 1, /* 128 query rows per workgroup (4 wavefronts x 32 rows), 2 workgroups per CU,
                             K/V tiles of 64 keys double-buffered in LDS                                */
  FA2_VARIANT_NARROW8 = 3 /* 256 query rows per workgroup (8 wavefronts x 32 rows), 1 workgroup per CU,
                             K/V loaded three tiles ahead, half the L2 -> LDS traffic per FLOP, no barrier
                             in the loop (the wavefronts count arrivals in LDS with one tile of slack);
                             when the Q tiles fill whole rounds of the CUs a workgroup takes one of every
                             round over one running K/V stream; needs N to be a multiple of 256 and
                             d <= 128.  FA2_VARIANT_AUTO takes it when the Q tiles fill whole rounds of
                             the 256 CUs (d = 128 also with very many tiles, and under the causal mask
                             from N = 2048 on) and the 128-row shape otherwise.  Its waits on the LDS
                             counters are bounded (tens of milliseconds): should a wavefront ever give
                             up, the rows it owns come out as NaN instead of the launch hanging         */
};

/*
 * fa2_fwd_variant -- fa2_fwd with an explicit tile shape, for tile-shape sweeps in the manner of the
 * paper's Table 1.  Arguments, layout, ownership and error behaviour are those of fa2_fwd; `variant`
 * is one of FA2_VARIANT_*.  An unknown variant is FA2_ERR_INVALID_ARG, a variant that cannot run the
 * shape is FA2_ERR_UNSUPPORTED.  All variants compute the same function; results may differ in the
 * last bits because the summation order differs.
 */
int fa2_fwd_variant(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N, int d,
                    float scale, int dtype, int variant, void* stream);

/* Masks of S. */
enum {
  FA2_MASK_NONE = 0,  /* every query attends to every key                                   */
  FA2_MASK_CAUSAL = 1 /* query i attends to keys j <= i only (autoregressive / decoder mask) */
};

/*
 * fa2_fwd_masked -- fa2_fwd with an optional mask applied to S before the softmax.  Section 2 of the
 * paper notes that entries of S may be set to -inf ahead of the row-wise softmax; FA2_MASK_CAUSAL does
 * so for every entry with key index j > query index i, so that
 *      O_i = softmax(scale * q_i . k_{0..i}) V_{0..i},     LSE[b,h,i] = ln sum_{j<=i} exp(scale * q_i . k_j).
 * Masked entries contribute exact zeros to P and to the row sum.  The kernel never loads K/V tiles that lie
 * wholly above the diagonal, so a causal call does about half the work of an unmasked one.
 *
 * Arguments, layout, ownership and error behaviour are those of fa2_fwd; `mask` is one of FA2_MASK_*
 * (anything else: FA2_ERR_INVALID_ARG).  FA2_MASK_NONE is exactly fa2_fwd.
 */
int fa2_fwd_masked(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N, int d,
                   float scale, int dtype, int mask, void* stream);

/*
 * fa2_fwd_qk -- the general shape of the Section 2 formula: Nq query rows attend to Nk keys and values
 * (the paper's SEQLEN and KEYLEN of Section 3), any Nq >= 1 and Nk >= 1.
 *
 *  Q        in   device, [B][Nq][H][d];   K, V  in  device, [B][Nk][H][d];
 *  O        out  device, [B][Nq][H][d];   LSE   out device, [B][H][Nq] fp32, may be NULL.
 *  mask          FA2_MASK_NONE, or FA2_MASK_CAUSAL, which needs Nq == Nk (FA2_ERR_UNSUPPORTED otherwise).
 *
 * Partial tiles are handled inside the kernel: columns of S that belong to keys past Nk-1 are set to
 * -inf before the softmax (exact zeros in P), rows past Nq-1 are never stored, and no byte outside the
 * four tensors is read or written.  Everything else -- layout within a row, element types, scale,
 * stream, ownership, error behaviour -- is as for fa2_fwd; fa2_fwd(…, N, …) is fa2_fwd_qk with
 * Nq = Nk = N and FA2_MASK_NONE.
 */
int fa2_fwd_qk(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int Nq, int Nk, int d,
               float scale, int dtype, int mask, void* stream);

/*
 * fa2_tile_shape -- which tile shape (FA2_VARIANT_NARROW or FA2_VARIANT_NARROW8) the entry points without a
 * `variant` argument use for a problem; the counterpart of reading the best cell off the paper's Table 1.  Host
 * only: nothing is launched and no HIP call is made.  Returns the FA2_VARIANT_* value (> 0), or a negative
 * FA2_ERR_* for sizes, head dimensions or masks that the entry points refuse.
 */
int fa2_tile_shape(int B, int H, int Nq, int Nk, int d, int mask);

/* Static, NUL-terminated description of a return code (never NULL). */
const char* fa2_strerror(int code);

/* Library version as major*10000 + minor*100 + patch. */
int fa2_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FA2_H_ */
