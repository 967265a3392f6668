/*
 * mdh.h -- C ABI of libmdh: tiled evaluation of multi-dimensional homomorphisms
 *
 *     md_hom(f, (op_1, ..., op_D))            (paper: Definition "Higher-Order Function md_hom")
 *
 * on one AMD MI355X (gfx950 / CDNA4).  A scalar function f is applied at every
 * point of a D-dimensional index space and dimension d is combined with op_d,
 * which is either concatenation (++) -- the dimension indexes the output -- or a
 * point-wise reduction operator (+, or the user-defined max-with-index).
 *
 * The library evaluates fixed instances of the paper's example table
 * (Figure "Data-parallel computations expressed in our high-level
 * representation"): MatMul, Jacobi-3D, multi-channel convolution (MCC), a
 * record-linkage style custom reduction, Dot, MatVec, the batched /
 * transposed MatMul variants and the row-wise scan; mdh_custom_* evaluates a
 * user-defined md_hom compiled at run time.  Each call takes the index-space sizes
 * N_1..N_D, the operand buffers the input/output views address, and one
 * configuration of the paper's tuning parameters (Table "Tuning parameters of
 * our low-level expressions"), restricted as in Section "Auto-Tuning".
 *
 * Conventions for every entry point
 *   - every buffer pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates, frees or synchronises; a call only enqueues kernels on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream);
 *     workspaces are cleared by kernels, not memsets, so a call may be captured
 *     into a HIP graph once one eager call with the same sizes and parameters
 *     has run on that device (the first use of a kernel sets its dynamic-LDS
 *     attribute and caches device properties; mdh_custom_run loads its module);
 *     the tune calls are the exception, they time candidates and synchronise;
 *   - inputs are never written; outputs are fully overwritten (the paper's
 *     re-composition overrides on first write, it does not accumulate into the
 *     destination: Appendix "Code Generation", re-composition phase);
 *   - all buffers are dense row-major (layout [1,2,...] in the paper's notation);
 *   - errors are reported through mdh_status only; an invalid call enqueues
 *     nothing; results are bit-identical run to run for fixed parameters.
 */
#ifndef MDH_H
#define MDH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mdh_status {
  MDH_OK = 0,
  MDH_ERR_NULL = 1,              /* a required pointer is NULL                                  */
  MDH_ERR_SIZE = 2,              /* a size is negative, a reduction extent is 0, or a buffer
                                    would exceed 2^31-1 elements                                */
  MDH_ERR_TILE_NOT_DIVIDING = 3, /* prod_l #PRT(l,d) * blk[d] != N_d (algorithmic constraint
                                    of tuning parameter 0)                                      */
  MDH_ERR_TILE_RESOURCES = 4,    /* model constraint violated: > 1024 lanes per workgroup,
                                    LDS or register budget exceeded                             */
  MDH_ERR_WORKSPACE = 5,         /* workspace missing or too small for a split reduction        */
  MDH_ERR_UNSUPPORTED = 6,       /* valid in the paper's space but no kernel instantiation      */
  MDH_ERR_LAUNCH = 7,            /* the HIP runtime refused the launch                          */
  MDH_ERR_STATIC_LIMIT = 8       /* mdh_custom_reduce_static: the call needs more scratch memory
                                    than the library's static buffer holds                      */
} mdh_status;

/* Instances (index into the library's table of md_hom expressions). */
typedef enum mdh_instance {
  MDH_MATMUL = 0,        /* md_hom(*, (++, ++, +)),            dims (i, j, k)              */
  MDH_STENCIL = 1,       /* md_hom(J_3D, (++, ++, ++)),        dims (i, j, k)              */
  MDH_MCC = 2,           /* md_hom(*, (++,++,++,++, +,+,+)),   dims (n, p, q, k, c, r, s)  */
  MDH_CUSTOM_REDUCE = 3, /* md_hom(wght, (++, max_idx)),       dims (a, b)                 */
  MDH_DOT = 4,           /* md_hom(*, (+)),                    dims (k)                    */
  MDH_MATVEC = 5,        /* md_hom(*, (++, +)),                dims (i, k)                 */
  MDH_BMATMUL = 6,       /* md_hom(*, (++, ++, ++, +)),        dims (b, i, j, k)           */
  MDH_SCAN = 7,          /* md_hom(id, (++, prefix-sum(+))),   dims (i, j)                 */
  MDH_MCC_CAPSULE = 8    /* md_hom(*, (++ x6, + x4)),  dims (n,p,q,k,mi,mj, c,r,s,mk)      */
} mdh_instance;

/*
 * Abstract System Model of the target (paper: Definition "Abstract System
 * Model"): ASM_CDNA4 = (3 memory layers, 3 core layers), the analogue of the
 * paper's ASM_CUDA+WRP.  Parts on a memory layer are processed sequentially,
 * parts on a core layer in parallel.
 */
enum {
  MDH_L_HBM = 0,  /* memory layer: sequential tiles streamed from device memory */
  MDH_L_LDS = 1,  /* memory layer: sequential tiles inside an LDS-resident tile  */
  MDH_L_VGPR = 2, /* memory layer: sequential elements inside a register tile    */
  MDH_L_WG = 3,   /* core layer: workgroups                                      */
  MDH_L_WAVE = 4, /* core layer: wavefronts (64 lanes) of a workgroup            */
  MDH_L_LANE = 5, /* core layer: lanes of a wavefront                            */
  MDH_NUM_LAYERS = 6,
  MDH_MAX_D = 10
};

/* Memory regions (parameters D3/S3/S5/R3). */
enum { MDH_MR_HBM = 0, MDH_MR_LDS = 1, MDH_MR_VGPR = 2 };

/*
 * One configuration of the tuning parameters, under the paper's own
 * restrictions (Section "Auto-Tuning": one fused loop nest, i.e. D1=S1=R1 and
 * D2=S2=R2; blocked or strided assignment only; full tiles per memory region).
 *
 * prt[l][d]  parameter 0, #PRT(l,d): number of parts of dimension d on layer l.
 * blk[d]     extent of the innermost block evaluated as one unit.  1 everywhere
 *            is the paper's full partitioning; the contractions use the FP32
 *            MFMA block (the coarser partitioning the paper names as future
 *            work for matrix hardware).  Constraint:
 *                prod_l prt[l][d] * blk[d] == N_d          (ragged == 0)
 *                prod_l prt[l][d] * blk[d] >= N_d          (ragged == 1; the
 *                tail parts are predicated -- an extension, the paper requires
 *                equality)
 * order[]    parameters D1=S1=R1: the fused loop order, outermost first, each
 *            entry = l * MDH_MAX_D + d; only the first MDH_NUM_LAYERS*D entries
 *            are used.  The layers come in one order in every kernel (workgroup parts,
 *            then device-memory tiles, wavefront and lane parts, LDS and register
 *            parts; returned by mdh_default_params).  A real choice inside the
 *            workgroup layer of MDH_MATMUL's LDS-tiled kernel: (WG,i) before (WG,j) =
 *            tiles dealt to the chip in bands of 8 tile rows, (WG,j) before (WG,i) =
 *            in bands of 8 tile columns (which panels of A and B the tiles that run
 *            together share).  Any other order has no instantiation:
 *            MDH_ERR_UNSUPPORTED.
 * strided    parameters D2=S2=R2 restricted to two values: 0 = blocked (outer
 *            parallelism: a core owns one contiguous part), 1 = strided.
 *            A real choice for MDH_DOT and MDH_MATVEC (lane assignment of the
 *            reduction dimension; both values run, blocked is the slow one) and for
 *            mdh_custom_* (walk order of the sequential parts), and for the few-channel
 *            kernel of MDH_MCC (blk[c] = 1): 0 = a workgroup owns a run of column tiles,
 *            1 = the tiles of (n, p, q) are dealt out one at a time, in arrival order, to
 *            the workgroups resident on the chip.  The other instances have one
 *            assignment per kernel and reject the other value.
 * lane_fast_dim  which md_hom dimension follows the fastest lane index (the
 *            paper's swizzle choice; decides coalescing).  A real choice for
 *            mdh_custom_* and for MDH_MATVEC (1 = lanes along k, the contiguous
 *            dimension of A: the default; 0 = lanes along i, a lane owns a row and walks
 *            all of k -- loads that do not coalesce, 5.6 times slower at 16384 x 16384);
 *            fixed per kernel elsewhere (the contiguous dimension).
 * in_region[b] / out_region   parameters D3/S3 and R3/S5: the fastest memory
 *            region input buffer b is staged in / results are combined in.  Real
 *            choices: MDH_MATMUL in_region LDS (wavefronts tile the output, operands
 *            staged in LDS) or VGPR (k on the wavefront layer, operands straight to
 *            registers, out_region = LDS); MDH_SCAN in_region VGPR (single pass) or
 *            HBM (three kernels); MDH_DOT and the small-M kernel of MDH_BMATMUL with
 *            a reduction split over workgroups: out_region HBM (the last workgroup
 *            part to arrive combines the parts in device memory, one launch) or VGPR
 *            (a second kernel does).  Other values: MDH_ERR_UNSUPPORTED.
 *
 * Counters inside the library.  The one-launch combination (out_region = MDH_MR_HBM) and
 * the dealt tiles of the few-channel MCC (strided = 1) count arrivals / hand out tickets
 * in small counter arrays that live in the library's device image; every launch leaves
 * them at zero.  Two such calls that overlap on one GPU (different streams or threads)
 * would share them: order such calls, or choose the other variant (out_region =
 * MDH_MR_VGPR, strided = 0), which uses nothing but the caller's buffers.
 * in_transposed[b] / out_transposed  parameters D4/S4, R4/S6 for 2-D tiles:
 *            for MDH_BMATMUL they are the views of the call (and must equal its
 *            flags); the other instances have plain layouts only.
 */
typedef struct mdh_tile_params {
  int32_t D;
  int32_t prt[MDH_NUM_LAYERS][MDH_MAX_D];
  int32_t blk[MDH_MAX_D];
  uint8_t order[MDH_NUM_LAYERS * MDH_MAX_D];
  uint8_t strided;
  uint8_t lane_fast_dim;
  uint8_t ragged;
  uint8_t in_region[4];
  uint8_t out_region;
  uint8_t in_transposed[4];
  uint8_t out_transposed;
  uint8_t reserved[3];
} mdh_tile_params;

/* ------------------------------------------------------------------------- */
/* Host-only helpers (no GPU needed)                                          */
/* ------------------------------------------------------------------------- */

/* Human-readable text for a status code; never NULL. */
const char* mdh_strerror(mdh_status s);

/* Runtime's text for the error behind the calling thread's most recent MDH_ERR_LAUNCH. */
const char* mdh_last_launch_error(void);

/* Library version, "major.minor". */
const char* mdh_version(void);

/*
 * Uniform MDA partitioning (paper: Appendix, Definition "MDA Partitioning").
 * For one dimension of extent N cut on L layers into P[0..L-1] parts, the part
 * addressed by p[0..L-1] starts at
 *     OS = sum_l p[l] * N / (P[0]*...*P[l])      and has      PS = N / prod_l P[l]
 * elements.  Returns MDH_ERR_TILE_NOT_DIVIDING unless prod_l P[l] divides N,
 * MDH_ERR_SIZE if some p[l] is outside [0,P[l]).
 */
mdh_status mdh_part_offset(int64_t N, int32_t L, const int32_t* P, const int32_t* p,
                           int64_t* offset, int64_t* part_size);

/*
 * The library's tuned default configuration for (instance, sizes).
 * `sizes` holds the D index-space extents in the dimension order listed at
 * mdh_instance; for MDH_MCC two more entries follow: stride_h, stride_w; for
 * MDH_CUSTOM_REDUCE one more entry follows: nF (read by mdh_tune only).
 * Host only; writes *out.
 */
mdh_status mdh_default_params(mdh_instance inst, const int64_t* sizes, mdh_tile_params* out);

/*
 * Check a configuration against the algorithmic constraint of parameter 0 and
 * the model constraints (paper: Appendix "Constraints of Programming Models":
 * at most 1024 lanes per workgroup; memory budgets), and against the set of
 * kernel instantiations this library has.  Host only, launches nothing.
 */
mdh_status mdh_validate_params(mdh_instance inst, const int64_t* sizes, const mdh_tile_params* p);

/*
 * Bytes of device workspace a call needs: non-zero only when a reduction
 * dimension is split over workgroups (prt[MDH_L_WG][d] > 1 for a non-++
 * dimension d), because workgroup results can only be combined in device
 * memory (paper: model constraint on R3 for the block layer).  params == NULL
 * means the default configuration.  Returns 0 on invalid arguments.
 */
size_t mdh_workspace_size(mdh_instance inst, const int64_t* sizes, const mdh_tile_params* params);

/* ------------------------------------------------------------------------- */
/* Device entry points                                                        */
/* ------------------------------------------------------------------------- */

/*
 * MatMul: C[i,j] = sum_k A[i,k] * B[k,j]  =  md_hom(*, (++,++,+)) with input
 * view (i,j,k)->A[i,k], (i,j,k)->B[k,j] and output view (i,j,0)->C[i,j]
 * (paper: Section "Examples", Subfigure 1).
 *   A: M x K, B: K x N, C: M x N, fp32, row-major, device.  K >= 1.
 *   M == 0 or N == 0 is a valid empty call.
 *   FP32 MFMA arithmetic, fp32 accumulation; if prt[MDH_L_WG][k] = S > 1 the
 *   S partial results go to `workspace` (S*M*N floats) and a second kernel adds
 *   them in ascending part order.  The library default may split k, so pass the
 *   workspace mdh_workspace_size asks for.  Two kernels, told apart in the table by
 *   prt[MDH_L_WAVE][k]: 1 = the wavefronts of a workgroup tile its output tile,
 *   operands staged in LDS (in_region = MDH_MR_LDS); WK > 1 = every wavefront owns
 *   the whole (small) output tile and 1/WK of the k-range, operands go straight to
 *   registers (in_region = MDH_MR_VGPR) and the WK results are added in LDS in
 *   ascending wavefront order (out_region = MDH_MR_LDS) -- the default for outputs
 *   of few tiles, blk = (16,16,4) or (32,32,2).  For M <= 16 mdh_matmul_ex (batch 1)
 *   has a kernel that streams B once and is several times faster still.
 */
mdh_status mdh_matmul(int64_t M, int64_t N, int64_t K, const float* A, const float* B, float* C,
                      const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * Jacobi-3D, one sweep of the 7-point stencil: md_hom(J_3D, (++,++,++)) whose
 * input view reads one buffer seven times with offset index functions (paper:
 * Section "Examples", Subfigure 4; 1-D form in Example "Input View -- Jacobi1D"):
 *   out[i,j,k] = c0*in[i+1,j+1,k+1] + c1*( in[i,j+1,k+1] + in[i+2,j+1,k+1]
 *              + in[i+1,j,k+1] + in[i+1,j+2,k+1] + in[i+1,j+1,k] + in[i+1,j+1,k+2] )
 *   in : (nx+2) x (ny+2) x (nz+2) fp32 (size rule N_buf = 1 + max index),
 *   out: nx x ny x nz fp32, compact (output view (i,j,k)->(i,j,k)).
 *   Any of nx, ny, nz == 0 is a valid empty call.
 */
mdh_status mdh_stencil(int64_t nx, int64_t ny, int64_t nz, const float* in, float* out, float c0,
                       float c1, const mdh_tile_params* params, void* stream);

/*
 * Multi-channel convolution: 7-dimensional md_hom(*, (++,++,++,++,+,+,+)) over
 * (n,p,q,k,c,r,s) with index functions p*stride_h+r, q*stride_w+s (paper:
 * Section "Examples", Subfigure 2; data characteristics table in the appendix):
 *   out[n,p,q,k] = sum_{c,r,s} in[n, p*stride_h + r, q*stride_w + s, c] * filt[k,r,s,c]
 *   in: N x H x W x C (NHWC), filt: K x R x S x C (KRSC), out: N x P x Q x K,
 *   P = (H-R)/stride_h + 1, Q = (W-S)/stride_w + 1 (no implicit padding),
 *   fp32, device.  C, R, S >= 1; H >= R; W >= S; strides >= 1.
 * Tile parameters: blk[p] x blk[q] is the pixel shape of the 32-pixel MFMA block
 * (1 x 32, 2 x 16 or 4 x 8), blk[k] = 32; blk[c] = 2 selects the channel-chunked
 * kernel, blk[c] = 1 the few-channel kernel that walks s and c as one dimension.
 * prt[MDH_L_WG][c] = S > 1 splits the reduction dimension c over workgroups: the S
 * partial outputs go to `workspace` (S * N*P*Q*K floats, see mdh_workspace_size) and
 * a second kernel adds them in ascending part order.  The library default does
 * that for small images with many channels, so pass the workspace
 * mdh_workspace_size asks for; it may be NULL when that size is 0.
 * Precondition of the few-channel kernel (blk[c] = 1, the default for C <= 8): the
 * input holds finite values.  Its fused (s,c) walk is padded to a multiple of 8 with
 * zero filter entries whose partners are real neighbouring input cells, and 0 * Inf
 * or 0 * NaN would put a NaN into an output whose own terms are all finite.
 */
mdh_status mdh_mcc(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R, int64_t S,
                   int64_t stride_h, int64_t stride_w, const float* in, const float* filt,
                   float* out, const mdh_tile_params* params, void* workspace,
                   size_t workspace_bytes, void* stream);

/*
 * Record-linkage style custom reduction: md_hom(wght, (++, max_idx)) over (a,b)
 * with an index-carrying scalar function (paper: Section "Examples",
 * Subfigure 5, and Appendix "Design Decisions: md_hom" for scalar functions
 * that receive MDA indices):
 *   wght(a,b)  = ( sum_f (A[a,f] == B[b,f] ? w_agree[f] : w_disagree[f]) , b )
 *   (s1,b1) max_idx (s2,b2) = the pair with the larger score; on equal scores
 *                             the pair with the smaller index
 *   out_score[a], out_index[a] = max_idx over all b.
 *   A: nA x nF, B: nB x nF, weights: nF, outputs: nA; all int32, device.
 *   1 <= nF <= 16, nB >= 1 (the operator has no neutral element), nA == 0 is an
 *   empty call.  The caller guarantees that no sum of nF weights overflows
 *   int32.  Integer arithmetic: the result is unique and reproduced bit-exactly.
 *   If B is split over workgroups (prt[MDH_L_WG][b] = S > 1) the S partial
 *   (score,index) pairs go to `workspace` (2*S*nA int32) and a second kernel
 *   combines them.
 */
mdh_status mdh_custom_reduce(int64_t nA, int64_t nB, int32_t nF, const int32_t* A,
                             const int32_t* B, const int32_t* w_agree, const int32_t* w_disagree,
                             int32_t* out_score, int32_t* out_index,
                             const mdh_tile_params* params, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * mdh_custom_reduce for callers that cannot allocate device memory -- code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments, results (bit for bit) and errors as mdh_custom_reduce, but
 * without the workspace arguments: the partial results of a reduction split over
 * workgroups (2 * S * nA int32, S = prt[MDH_L_WG][b]) go to a static device array
 * inside the library, mdh_static_scratch_bytes() = 16 MiB per GPU, which the GPU
 * holds until the process ends.  A call whose partial results do not fit returns
 * MDH_ERR_STATIC_LIMIT and enqueues nothing (at the default configuration of
 * 2^16 x 2^18 records, S = 32, they fit exactly); pass a configuration with a
 * smaller S, or use mdh_custom_reduce with a workspace.  The call allocates and
 * frees nothing and synchronises nothing; the first call on a device looks up the
 * array's device address.  All calls on one GPU share that array: calls that may
 * overlap (different streams, or threads) race on it and must be ordered by the
 * caller; calls on one stream are ordered by the stream.
 */
mdh_status mdh_custom_reduce_static(int64_t nA, int64_t nB, int32_t nF, const int32_t* A,
                                    const int32_t* B, const int32_t* w_agree,
                                    const int32_t* w_disagree, int32_t* out_score,
                                    int32_t* out_index, const mdh_tile_params* params, void* stream);
/* Size in bytes of the static scratch array of mdh_custom_reduce_static (host only). */
size_t mdh_static_scratch_bytes(void);

/*
 * MCC_Capsule: MCC on 4 x 4 matrices instead of scalars,
 *   out[n,p,q,k,mi,mj] = sum_{c,r,s,mk} in[n, p*stride_h+r, q*stride_w+s, c, mi, mk]
 *                                        * filt[k, r, s, c, mk, mj]
 * = md_hom(*, (++,++,++,++,++,++, +,+,+,+)) over (n,p,q,k,mi,mj,c,r,s,mk) (paper:
 * Section "Examples", Subfigure 2; Appendix "Data Characteristics used in Deep
 * Neural Networks": MCC with three more dimensions MI = MJ = MK = 4).
 *   in:   N x H x W x C x 4 x 4        filt: K x R x S x C x 4 x 4
 *   out:  N x P x Q x K x 4 x 4,  P, Q as for mdh_mcc; all fp32, dense, device.
 * The whole filter slice of a workgroup is staged in LDS: shapes whose slice
 * (8 channels x R x S x C x 16 floats) plus input patch exceed 160 KB are refused
 * with MDH_ERR_TILE_RESOURCES (few input channels, as in the paper's study).
 * `sizes` for the host helpers: (N, P, Q, K, C, R, S, stride_h, stride_w).
 */
mdh_status mdh_mcc_capsule(int64_t N, int64_t H, int64_t W, int64_t C, int64_t K, int64_t R,
                           int64_t S, int64_t stride_h, int64_t stride_w, const float* in,
                           const float* filt, float* out, const mdh_tile_params* params,
                           void* stream);

/*
 * Row-wise scan: out[i,j] = in[i,0] + ... + in[i,j]  =  md_hom(id, (++, prefix-sum(+)))
 * over (i,j) (paper: Section "Examples", Subfigure 8; combine operator: Appendix,
 * Example "Prefix-Sum").  The prefix-sum operator keeps the dimension and a part
 * needs ONE value of the parts before it (their last prefix); that value is
 * passed lane -> wavefront (registers) -> workgroup (LDS) -> sequential tiles
 * (a carry; rows of up to 8 tiles can instead stay in registers as register-layer
 * parts) -> and, if prt[MDH_L_WG][j] = C > 1, across workgroups, in one of
 * two ways that the table tells apart by in_region[0]:
 *   MDH_MR_VGPR  single pass: a chunk (1, 2, 4 or 8 tiles, register-layer parts:
 *                prt[MDH_L_VGPR][j] = 4 * tiles, prt[MDH_L_HBM][j] = 1) waits in registers while
 *                the workgroups exchange chunk totals, and sums of 64 totals,
 *                through `workspace`; 8 bytes of HBM traffic per element.  Chunk
 *                numbers are handed out in the order in which workgroups start,
 *                so a workgroup only waits for workgroups that already run; each
 *                wait is bounded, and should a bound ever be hit the kernel stops
 *                waiting, finishes with wrong values in that chunk and sets the
 *                second 8-byte word of `workspace` to 1 (0 otherwise).
 *   MDH_MR_HBM   three kernels: chunk totals, their exclusive scan per row, then
 *                every chunk scanned from its offset; the input is read twice
 *                (12 bytes per element).
 * Both add in a fixed order (bit-identical run to run).  `workspace`: 8-byte
 * aligned, mdh_workspace_size() bytes (R*C doubles for three kernels;
 * 2 + R*C + R*ceil(C/64) 8-byte words for the single pass); its contents need no
 * initialisation and calls that share it must be ordered on one stream.
 *   in, out: R x n fp32, row-major, device; may not overlap.  R == 0 or n == 0 is
 *   an empty call.  `sizes` for the host helpers: (R, n).
 */
mdh_status mdh_scan(int64_t R, int64_t n, const float* in, float* out,
                    const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                    void* stream);

/*
 * Did a bounded wait of the single-pass scan expire in the last mdh_scan call that used
 * `workspace` with these sizes and parameters?  Synchronises `stream` (pass the stream of
 * that call), then reads the flag word of the workspace: *timed_out = 1 means the output
 * of that call is wrong in at least one chunk and must be discarded (the scan of the paper's
 * Example "Prefix-Sum" has no such failure mode; it belongs to this single-pass kernel).
 * Configurations without waits (one chunk per row, or three kernels) always report 0.
 * Host call; not for use under graph capture.
 */
mdh_status mdh_scan_timed_out(int64_t R, int64_t n, const mdh_tile_params* params, const void* workspace,
                              void* stream, int32_t* timed_out);

/*
 * Dot product: out = sum_k x[k] * y[k]  =  md_hom(*, (+)) over (k) with output
 * view (0) -> the scalar `out` (paper: Section "Examples", Subfigure 1, first
 * routine).  The only dimension is a reduction: it is split over lanes
 * (combined across the wavefront in registers), wavefronts (combined in LDS)
 * and, if prt[MDH_L_WG][k] = S > 1, workgroups (S partial sums in `workspace`,
 * S floats, combined by a second kernel in ascending part order).
 *   x, y: K fp32 each, device; out: 1 fp32, device.  K >= 1.
 */
mdh_status mdh_dot(int64_t K, const float* x, const float* y, float* out,
                   const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                   void* stream);

/*
 * Matrix-vector product: y[i] = sum_k A[i,k] * x[k]  =  md_hom(*, (++, +)) over
 * (i,k) with views (i,k)->A[i,k], (i,k)->x[k], (i,0)->y[i] (paper: the
 * introductory example, and the worked example of Section "Low-Level
 * Representation").  k is the contiguous dimension of A and runs over the lanes,
 * so the reduction is re-composed lane -> wavefront -> workgroup -> (if
 * prt[MDH_L_WG][k] = S > 1) grid through `workspace` (S*M floats).
 *   A: M x K, x: K, y: M, fp32, row-major, device.  K >= 1; M == 0 is an empty call.
 */
mdh_status mdh_matvec(int64_t M, int64_t K, const float* A, const float* x, float* y,
                      const mdh_tile_params* params, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * Batched MatMul with transposed views: bMatMul = md_hom(*, (++,++,++,+)) over
 * (b,i,j,k); MatMul^T is the same md_hom with other index functions (paper:
 * Section "Examples", Subfigure 1, routines 4 and 5):
 *   C_b[i,j] = sum_k A_b[i,k] * B_b[k,j]   for every batch entry b < batch
 *   trans_a: A_b is stored K x M and read through (b,i,j,k)->A[b,k,i]
 *   trans_b: B_b is stored N x K and read through (b,i,j,k)->B[b,j,k]
 *   trans_c: C_b is stored N x M, written through (b,i,j,0)->C[b,j,i]
 * All buffers dense, batch-major, fp32, device.  K >= 1; batch, M or N == 0 is an
 * empty call; batch <= 65535.  Split reductions need batch*S*M*N floats of workspace.
 * For mdh_default_params etc. the `sizes` of MDH_BMATMUL are
 * (batch, M, N, K, trans_a, trans_b, trans_c); a configuration's in_transposed[0..1]
 * and out_transposed must equal the call's flags.
 * Two kernels: blk = (1,32,32,2), LDS-tiled, any views; blk = (1,16,16,4) for M <= 16
 * with A and C plain (B plain or transposed), which streams both operands from
 * device memory straight into MFMA operand registers and parallelises k over
 * wavefronts and workgroups (the library default for those shapes).  That kernel
 * has two strip widths: prt[MDH_L_VGPR][j] = 4 (a wavefront owns 64 columns; k may
 * be split over workgroups, combined as out_region says) and prt[MDH_L_VGPR][j] = 1
 * (a workgroup owns 16 columns and all of k: prt[MDH_L_WG][k] = 1, 8 or 16
 * wavefronts along k, no workspace).  With trans_b the 16-column strips also exist
 * with in_region[0..1] = MDH_MR_LDS (4 or 8 wavefronts along k): rows of A and B are
 * read as whole runs of k and reach the MFMA operand layout through LDS; the default
 * for trans_b when the strips fill the chip or K <= 3072.
 */
mdh_status mdh_matmul_ex(int64_t batch, int64_t M, int64_t N, int64_t K, const float* A,
                         int32_t trans_a, const float* B, int32_t trans_b, float* C,
                         int32_t trans_c, const mdh_tile_params* params, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * Small per-workload tile-parameter search (paper: Section "Auto-Tuning", with
 * the search space shrunk to this library's kernel instantiations): runs every
 * valid candidate for (instance, sizes) on the given buffers, times each with
 * events on `stream`, and writes the fastest configuration to *best and its
 * time to *best_ms.  `buffers` are the device pointers of the instance's entry
 * point in declaration order (inputs then outputs); outputs are overwritten.
 * `scalars` carries c0,c1 for the stencil and is ignored otherwise.
 * Synchronises `stream`.  Not for use under graph capture.
 */
mdh_status mdh_tune(mdh_instance inst, const int64_t* sizes, void* const* buffers,
                    const float* scalars, void* workspace, size_t workspace_bytes, void* stream,
                    int32_t reps, mdh_tile_params* best, float* best_ms);

/*
 * Number of candidate configurations mdh_tune would try for (instance, sizes),
 * and the idx-th of them (host only).
 */
int32_t mdh_num_candidates(mdh_instance inst, const int64_t* sizes);
mdh_status mdh_candidate(mdh_instance inst, const int64_t* sizes, int32_t idx,
                         mdh_tile_params* out);

/* ------------------------------------------------------------------------- */
/* Generic md_hom with runtime-compiled scalar function and combine operator  */
/* ------------------------------------------------------------------------- */
/*
 * The method itself rather than a fixed instance (paper: Definition "Higher-Order
 * Function md_hom", Definitions "Input View" / "Output View"; Section
 * "Experimental Results" on user-defined scalar types and operators, e.g. PRL):
 *
 *   out[out_index(i)] = op_1 ... op_D  f( in_{b_1}[idx_1(i)], ..., in_{b_A}[idx_A(i)], i )
 *
 * with op_d = ++ (reduce[d] = 0), op_d = pw(op) (reduce[d] = 1) or, for at most
 * one dimension, op_d = prefix-sum(op) (reduce[d] = 2; paper: Appendix, Example
 * "Prefix-Sum": the dimension is kept and index i holds the combination of all
 * indices <= i; this kernel walks it sequentially per lane), a user-defined
 * result type T, scalar function f and operator op given as C source and compiled
 * for gfx950 when the operation is created (hipRTC).  All point-wise dimensions of
 * one operation share ONE operator op, which must be associative and commutative
 * (paper: Lemma on mixes of ++ and pw); no neutral element is needed (the first
 * value of a part overrides).  The index functions may read one buffer several
 * times (stencils) and are arbitrary C expressions (views).
 *
 * Source conventions.  Every string is C/HIP device code:
 *   prelude      type definitions and helper functions, placed first (may be NULL)
 *   in_type[b]   element type of input buffer b (e.g. "float", or a struct of prelude)
 *   acc_buf[a], acc_index[a]
 *                access a reads buffer acc_buf[a] at the flat element index given by
 *                the expression acc_index[a] over i0..i{D-1} (type long long) and
 *                the sizes N0..N{D-1}: index function composed with the row-major
 *                layout of the buffer
 *   out_type     T: type of f's result, of op's operands and of the output elements
 *   out_elem_bytes  sizeof(T), checked against the compiled code
 *   out_index    flat element index in the output buffer; NULL = row-major over the
 *                ++ (and prefix-sum) dimensions.  Indices of reduced dimensions are 0.
 *   f            statements that set `T r` from a0..a{A-1} (the accessed elements,
 *                const references) and i0..i{D-1}
 *   op           statements that set `T r` from `x` and `y` (const T references)
 *   fast_dim     dimension whose consecutive indices are consecutive in memory for
 *                the largest operand (gets the fastest lane index); -1 = D-1
 *
 * De-composition.  Every dimension is cut into #PRT(WG,d) workgroup parts x
 * #PRT(LANE,d) lane parts x #PRT(HBM,d) sequential parts x #PRT(VGPR,d) register
 * parts (blk = 1: the paper's full partitioning; inputs stay in device memory).
 * Register parts exist for ++ dimensions only: a lane then holds
 * prod #PRT(VGPR,d) results at once, and an input element whose index function does
 * not use a register-blocked dimension is loaded once for all of its parts.
 * `strided` = 1: index = ((q*WG + g)*LANE + l)*VGPR + v; 0: ((g*Q + q)*LANE + l)*VGPR + v.
 * Re-composition: registers -> LDS tree over the lanes of the reduced dimensions
 * -> workspace + second kernel over their workgroup parts, every level in a fixed
 * order (deterministic).  mdh_custom_default_params / mdh_custom_candidate supply
 * configurations; explicit ones are validated like those of the fixed instances
 * (MDH_ERR_TILE_NOT_DIVIDING, MDH_ERR_TILE_RESOURCES, also when a workgroup part
 * of a reduced dimension would be empty).
 *
 * mdh_custom_create compiles (host only: works without a GPU) and returns an
 * operation handle; `log` (may be NULL) receives the compiler's messages.  The
 * first mdh_custom_run of a handle loads the code object on the current device (the
 * only allocation the runtime makes on behalf of this library; a handle stays with
 * that device); after that a run only enqueues one or two kernels.  inputs[b] / output / workspace are device pointers; the workspace
 * needs mdh_custom_workspace_size(op) bytes (0 if no reduced dimension is split
 * over workgroups).  Runs of one handle may be issued from several threads; create
 * and destroy are the caller's to order.
 * Errors: MDH_ERR_NULL, MDH_ERR_SIZE (D, n_in, n_acc, sizes out of range),
 * MDH_ERR_UNSUPPORTED (source does not compile: see log), MDH_ERR_WORKSPACE,
 * MDH_ERR_LAUNCH, and the tile errors above.
 */
#define MDH_CUSTOM_MAX_IN 4
#define MDH_CUSTOM_MAX_ACC 8
typedef struct mdh_custom_desc {
  int32_t D;
  int64_t sizes[MDH_MAX_D];
  uint8_t reduce[MDH_MAX_D];
  int32_t n_in;
  int32_t n_acc;
  int32_t acc_buf[MDH_CUSTOM_MAX_ACC];
  int32_t out_elem_bytes;
  int32_t fast_dim;
  const char* prelude;
  const char* in_type[MDH_CUSTOM_MAX_IN];
  const char* acc_index[MDH_CUSTOM_MAX_ACC];
  const char* out_type;
  const char* out_index;
  const char* f;
  const char* op;
} mdh_custom_desc;

typedef struct mdh_custom_op mdh_custom_op;

mdh_status mdh_custom_default_params(const mdh_custom_desc* desc, mdh_tile_params* out);
mdh_status mdh_custom_validate_params(const mdh_custom_desc* desc, const mdh_tile_params* params);
int32_t mdh_custom_num_candidates(const mdh_custom_desc* desc);
mdh_status mdh_custom_candidate(const mdh_custom_desc* desc, int32_t idx, mdh_tile_params* out);
mdh_status mdh_custom_create(const mdh_custom_desc* desc, const mdh_tile_params* params,
                             mdh_custom_op** out, char* log, size_t log_bytes);
/* Generated device source of the operation (owned by the handle; never NULL). */
const char* mdh_custom_source(const mdh_custom_op* op);
size_t mdh_custom_workspace_size(const mdh_custom_op* op);
mdh_status mdh_custom_run(mdh_custom_op* op, const void* const* inputs, void* output,
                          void* workspace, size_t workspace_bytes, void* stream);
void mdh_custom_destroy(mdh_custom_op* op);
/*
 * The small search for the generic path: compiles the first `max_candidates`
 * candidate configurations of `desc` (<= 0: all of them, a second or so each),
 * runs each `reps` times on the given device buffers (the output is overwritten)
 * and returns the fastest and its milliseconds per run.  Candidates that need
 * more workspace than given are skipped.  Synchronises `stream`.
 */
mdh_status mdh_custom_tune(const mdh_custom_desc* desc, const void* const* inputs, void* output,
                           void* workspace, size_t workspace_bytes, void* stream, int32_t reps,
                           int32_t max_candidates, mdh_tile_params* best, float* best_ms);

/* ------------------------------------------------------------------------- */
/* Calibration kernels (measurement support; nothing of the method)           */
/* ------------------------------------------------------------------------- */
/*
 * What the chip attains on the resources the instances are bound by, with
 * nothing else in the way: a roofline fraction quoted against the published
 * peak (paper: Section "Experimental Results" measures against hand-tuned
 * libraries instead) can then be read against the attainable rate as well.
 * Every call enqueues one kernel (the arithmetic ones MDH_CALIB_BLOCKS workgroups x
 * 256 lanes; the streaming read one workgroup of 512 lanes per compute unit, the copy
 * one workgroup of 256 lanes per 16 KB piece: the launch shapes measured fastest).
 *   mdh_calib_copy : dst[0..bytes) = src[0..bytes), 16-byte non-temporal accesses;
 *                    bytes > 0 and a multiple of 16, both pointers 16-byte aligned.
 *   mdh_calib_read : streams src once; the first MDH_CALIB_STREAM_LANES floats of
 *                    `out` (device) receive one partial sum per lane.
 *   mdh_calib_mfma : every wavefront issues iters*16 independent
 *                    v_mfma_f32_32x32x2_f32; *flop (host, may be NULL) receives the
 *                    floating-point operations of the launch; `out` as above.
 *   mdh_calib_valu : every lane issues iters*64 plain 32-bit integer VALU
 *                    instructions; *lane_ops (host, may be NULL) receives lanes x
 *                    instructions; `out`: MDH_CALIB_BLOCKS*256 int32 (device).
 * Errors: MDH_ERR_NULL, MDH_ERR_SIZE, MDH_ERR_LAUNCH.
 */
#define MDH_CALIB_BLOCKS 2048
#define MDH_CALIB_STREAM_LANES (256 * 512)
mdh_status mdh_calib_copy(const void* src, void* dst, int64_t bytes, void* stream);
mdh_status mdh_calib_read(const void* src, int64_t bytes, float* out, void* stream);
mdh_status mdh_calib_mfma(float* out, int32_t iters, int64_t* flop, void* stream);
mdh_status mdh_calib_valu(int32_t* out, int32_t iters, int64_t* lane_ops, void* stream);

/*
 * Integer VALU issue rate by instruction kind, with the shader clock read beside it
 * (the ceiling the custom reduce is measured against; paper: Section "Examples",
 * Subfigure 5 is the instance, its inner loop is what these loops are made of).
 * Every kernel is a register-resident loop of MDH_CALIB_BLOCKS workgroups x 256 lanes,
 * eight independent chains per lane, issuing ONE kind of instruction:
 *   MDH_CALIB_KIND_XOR_MAX     v_xor + v_max pairs (the loop of mdh_calib_valu)
 *   MDH_CALIB_KIND_CMP_SELECT  compare against a scalar-register operand + select
 *   MDH_CALIB_KIND_ADD3        three-operand add
 *   MDH_CALIB_KIND_FMA_F32     fp32 fused multiply-add on vector-register operands
 *   MDH_CALIB_KIND_ADD_VGPR    32-bit add on vector-register operands (these two are of
 *                              the kind the vector ALU issues at 32 lanes a cycle)
 *   MDH_CALIB_KIND_PRL_MIX     the custom reduce's own inner loop at nF = 8 and two
 *                              records of A per lane (per pair: 8 compares against a
 *                              scalar operand, 8 selects, 4.5 adds, compare + max +
 *                              select + half a move = 24 instructions), with the
 *                              records of B made up on the scalar unit, not loaded
 *   MDH_CALIB_KIND_PRL_FAST_MIX the custom reduce's loop for 8 fields as built from the
 *                              fast kinds (per pair: 8 x (fp32 subtract, multiply with
 *                              clamp, fused multiply-add), and per block of four records
 *                              of B two three-operand maxima, a compare and a select),
 *                              one trip = one block = 8 pairs = 203 instructions
 *   out      MDH_CALIB_BLOCKS*256 int32 (device), overwritten
 *   weights  the two PRL kinds only (else may be NULL): MDH_CALIB_MIX_WEIGHTS int32 (device):
 *            8 agree weights, 8 disagree weights, then 256 lanes x 2 records x 8 fields
 *   iters    loop trips; *lane_ops (host, may be NULL) receives lanes x VALU instructions
 *            issued inside the loops of the launch
 *   clocks   device, 2 x int64, may be NULL: the first wavefront of workgroup 0 writes
 *            the shader-clock cycles and the constant-rate real-time ticks
 *            (mdh_calib_realtime_hz() per second) that passed around its loop, so
 *            shader clock = clocks[0] / clocks[1] * mdh_calib_realtime_hz()
 * Errors: MDH_ERR_NULL, MDH_ERR_SIZE, MDH_ERR_UNSUPPORTED (kind), MDH_ERR_LAUNCH.
 */
enum {
  MDH_CALIB_KIND_XOR_MAX = 0,
  MDH_CALIB_KIND_CMP_SELECT = 1,
  MDH_CALIB_KIND_ADD3 = 2,
  MDH_CALIB_KIND_PRL_MIX = 3,
  MDH_CALIB_KIND_FMA_F32 = 4,
  MDH_CALIB_KIND_ADD_VGPR = 5,
  MDH_CALIB_KIND_PRL_FAST_MIX = 6
};
#define MDH_CALIB_MIX_WEIGHTS (16 + 256 * 2 * 8)
mdh_status mdh_calib_valu_kind(int32_t kind, int32_t* out, const int32_t* weights, int32_t iters,
                               int64_t* lane_ops, int64_t* clocks, void* stream);
/* Rate of the real-time counter of the current device in Hz (host only; 0 if unknown). */
int64_t mdh_calib_realtime_hz(void);

#ifdef __cplusplus
}
#endif
#endif /* MDH_H */
