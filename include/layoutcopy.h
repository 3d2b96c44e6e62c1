/* layoutcopy.h — C ABI of the MI355X (gfx950) layout-algebra and layout-driven tensor copy library.
 *
 * Vocabulary follows "CuTe Layout Representation and Algebra":
 *   - a Layout is a congruent pair Shape:Stride of hierarchical tuples of integers (Sec. 2.3-2.4) and
 *     is a function from coordinates to offsets: L(c) = inner_product(idx2crd_S(c), D)
 *     (Eq. idx2crd, Eq. innerprod, Sec. 2.4 Def. layout);
 *   - a Tensor is a pointer accessor composed with a layout, T(c) = *(e + L(c)) (Sec. 2.5, Eq. tensor);
 *   - COPY moves dst(i) = src(i) for every integral coordinate i (Sec. 2.6.1).
 *
 * Conventions that hold for every entry point
 *   - Strides and offsets are counted in ELEMENTS of the copy's dtype, never in bytes.  Strides are integers of either
 *     sign (Sec. 2.3.2: Z is an integer-semimodule): the layout function, coalesce, slicing and COPY take negative
 *     strides; the operations whose statements are written for strides in N return NEGATIVE_STRIDE for them.
 *   - Layout and plan handles are host objects, immutable after creation, owned by the caller and
 *     released with the matching destroy call.  Handles may be shared between threads.
 *   - `const void* src` / `void* dst` of the copy calls are DEVICE pointers to offset 0 of the
 *     respective layout; the caller owns that memory and guarantees that the offsets
 *     [min_offset(layout), cosize(layout)) around it are addressable.  The library allocates no device memory, never synchronises the device and
 *     launches only on the stream it is given (`hip_stream` is a hipStream_t passed as void*;
 *     NULL = the default stream).
 *   - Every call returns an lc_status_t; on error `*out` is left untouched.  No C++ exception
 *     crosses this boundary.
 */
#ifndef LAYOUTCOPY_H_
#define LAYOUTCOPY_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lc_layout lc_layout_t; /* opaque: a layout S:D */
typedef struct lc_plan lc_plan_t;     /* opaque: a planned copy between two layouts */
typedef struct lc_slayout lc_slayout_t; /* opaque: a layout whose strides come from an integer-semimodule (Sec. 2.3.2) */
typedef struct lc_gemm_plan lc_gemm_plan_t; /* opaque: a planned GEMM over three layouts */

typedef enum {
  LC_OK = 0,
  LC_ERR_INVALID_ARG = 1,         /* NULL where a handle/pointer is required, bad rank, bad cotarget ... */
  LC_ERR_PARSE = 2,               /* text is not "S:D" in the paper's notation */
  LC_ERR_NOT_CONGRUENT = 3,       /* shape and stride have different profiles (Sec. 2.3: S ~ D) */
  LC_ERR_BAD_EXTENT = 4,          /* an extent < 1 (a shape is an HTuple of positive integers, Sec. 2.2) */
  LC_ERR_NEGATIVE_STRIDE = 5,     /* an operation stated for strides in N (composition, complement, inverses, divides, products, GEMM) was given a negative stride */
  LC_ERR_SIZE_MISMATCH = 6,       /* COPY precondition size(src) == size(dst) violated (Sec. 2.6.1) */
  LC_ERR_STRIDE_DIVISIBILITY = 7, /* composition: stride divisibility condition (Eq. divis_stride) */
  LC_ERR_SHAPE_DIVISIBILITY = 8,  /* composition: shape divisibility condition (Eq. divis_shape) */
  LC_ERR_NOT_SEGREGATED = 9,      /* composition: sublayouts of B without segregated images (Sec. 3.3.2) */
  LC_ERR_NOT_INJECTIVE = 10,      /* complement: a mode of the layout overlaps the span of smaller ones */
  LC_ERR_NOT_SURJECTIVE = 11,     /* logical divide: (B, B*) misses coordinates of A (Sec. 3.5.2) */
  LC_ERR_DST_ALIASES = 12,        /* GEMM: two coordinates of C share an offset (copies with such a destination plan as "last-writer") */
  LC_ERR_UNSUPPORTED_DTYPE = 13,
  LC_ERR_TOO_LARGE = 14,          /* size or cosize beyond 2^62, more than 64 leaf modes, or more work than the kernels index */
  LC_ERR_MISALIGNED = 15,         /* a device pointer is less aligned than the plan was created for */
  LC_ERR_HIP = 16,                /* a HIP runtime call failed (no device, launch failure, ...) */
  LC_ERR_NEEDS_WORKSPACE = 17,    /* the plan needs scratch device memory: use lc_plan_execute_workspace */
  LC_ERR_WORKSPACE_TOO_SMALL = 18,/* the workspace is NULL, misaligned or smaller than lc_plan_workspace_bytes */
  LC_ERR_SCRATCH_LIMIT = 19       /* lc_plan_execute_static: the plan needs more scratch than the library's static array holds */
} lc_status_t;

/* Element types.  The copy moves bit patterns; the dtype only fixes the element width. */
typedef enum {
  LC_F32 = 0, LC_F16 = 1, LC_BF16 = 2,
  LC_B8 = 3, LC_B16 = 4, LC_B32 = 5, LC_B64 = 6, LC_B128 = 7 /* opaque elements of 1, 2, 4, 8, 16 bytes */
} lc_dtype_t;

const char* lc_status_string(lc_status_t s);
/* Text of the HIP error behind the calling thread's most recent LC_ERR_HIP ("" if there was none).
 * The pointer stays valid until the thread's next failing call. */
const char* lc_last_hip_error(void);
int lc_dtype_bytes(lc_dtype_t dt); /* element width in bytes, 0 for an unknown dtype */

/* ---------------------------------------------------------------------------------------------
 * Layout construction and inspection (Sec. 2.1-2.4)
 * ------------------------------------------------------------------------------------------- */

/* Parse the paper's printed form, e.g. "((8,512),(8,1024)):((1,8),(4096,32768))" or "24:3"
 * (Sec. 2.4.1).  Whitespace is ignored; strides may be negative.  Errors: PARSE, NOT_CONGRUENT, BAD_EXTENT, TOO_LARGE. */
lc_status_t lc_layout_parse(const char* text, lc_layout_t** out);

/* Build from a pre-order encoding of the shape tree: an entry -k (k >= 1) opens a tuple of k children,
 * a positive entry is a leaf extent.  `leaf_strides` lists the strides of the leaves left to right
 * (host arrays, copied). */
lc_status_t lc_layout_from_tree(const int64_t* shape_preorder, int n_nodes, const int64_t* leaf_strides,
                                int n_leaves, lc_layout_t** out);
void lc_layout_destroy(lc_layout_t* layout);

/* Writes the printed form into buf (NUL-terminated, truncated to cap); *needed (optional) receives the
 * size including the terminator. */
lc_status_t lc_layout_to_string(const lc_layout_t* layout, char* buf, size_t cap, size_t* needed);

int64_t lc_layout_size(const lc_layout_t* layout);   /* |L|: product of the extents (Sec. 2.4.1) */
int64_t lc_layout_cosize(const lc_layout_t* layout); /* largest offset of the image + 1 (Sec. 2.4.1) */
int64_t lc_layout_min_offset(const lc_layout_t* layout); /* smallest offset of the image: 0 unless a stride is negative */
int lc_layout_rank(const lc_layout_t* layout);       /* Sec. 2.1 */
int lc_layout_depth(const lc_layout_t* layout);      /* Sec. 2.1 */

/* L(i) for an integral coordinate.  Any i >= 0 is accepted: beyond |L| the last mode is left
 * unreduced (extended domain, Sec. 2.2.2 and 2.4.1). */
int64_t lc_layout_eval(const lc_layout_t* layout, int64_t integral_coord);

/* Slicing (Sec. 2.5.1): `coord` is a coordinate in the paper's notation with "_" at the unspecified
 * positions, e.g. "(2,((0,_),_))"; an integer may stand for a whole sub-mode (integral coordinate of
 * that mode).  *offset receives L(specified part) — add it to the tensor's pointer — and *out the
 * sublayout of the unspecified modes ("1:0" if none is left).  Errors: PARSE, NOT_CONGRUENT. */
lc_status_t lc_layout_slice(const lc_layout_t* layout, const char* coord, int64_t* offset, lc_layout_t** out);

/* ---------------------------------------------------------------------------------------------
 * Layout algebra (Sec. 3).  Each call allocates *out on LC_OK.
 * A tiler (Sec. 3.3.5) is passed as a layout whose top-level modes are the tiles; an integer tile S is
 * the mode S:1.  A layout whose shape is a single integer is the 1-tuple tiler of itself.
 * ------------------------------------------------------------------------------------------- */

/* Coalesce (Sec. 3.2): depth <= 1, same size, same value at every integral coordinate; extent-1
 * modes removed, neighbouring modes merged when stride_{k+1} = extent_k * stride_k; "1:0" if nothing is left. */
lc_status_t lc_coalesce(const lc_layout_t* a, lc_layout_t** out);
/* Coalesce applied to every top-level mode separately (Sec. 3.2, Eq. layout_combinator). */
lc_status_t lc_coalesce_bymode(const lc_layout_t* a, lc_layout_t** out);

/* Group composition R = A o B (Sec. 3.3): B's shape is compatible with R's and R(c) = A(B(c)) for
 * every coordinate of B.  Errors: STRIDE_DIVISIBILITY, SHAPE_DIVISIBILITY, NOT_SEGREGATED. */
lc_status_t lc_composition(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out);
/* By-mode composition with a tiler (Sec. 3.3.5): (A_0 o T_0, A_1 o T_1, ...); modes of A beyond the
 * tiler's rank are kept whole. */
lc_status_t lc_composition_bymode(const lc_layout_t* a, const lc_layout_t* tiler, lc_layout_t** out);

/* Complement (Sec. 3.5) with respect to `cotarget` offsets (0 = cosize(a)): ordered image, disjoint
 * from the image of `a` on its whole extended domain; ends with the mode that steps over everything
 * (e.g. "1:32").  Errors: NOT_INJECTIVE, INVALID_ARG (cotarget < 0). */
lc_status_t lc_complement(const lc_layout_t* a, int64_t cotarget, lc_layout_t** out);

/* Right-inverse of maximal size (Sec. 3.4.1): injective, a(out(k)) = k for every k < |out|; "1:0" when trivial. */
lc_status_t lc_right_inverse(const lc_layout_t* a, lc_layout_t** out);

/* Left-inverse (Sec. 3.4.3): a(out(a(k))) = a(k) for every k < |a|, and out(a(k)) = k when `a` is
 * injective.  Stride-0 modes of `a` are not inverted.  Errors: NOT_INJECTIVE (moving modes overlap),
 * STRIDE_DIVISIBILITY (a stride does not divide the next larger one: no layout inverts that). */
lc_status_t lc_left_inverse(const lc_layout_t* a, lc_layout_t** out);
/* Application of the left-inverse (Sec. 3.4.3): does the data layout `a` hold every offset the instruction layout `t`
 * accesses, i.e. is there for every i < |t| a coordinate c of `a` with t(i) = a(c)?  Decided as the paper does, by
 * a(a^†(t(i))) = t(i) with a^†(t(i)) inside a's domain.  *yes receives 1 or 0.  `where` (optional): on yes, *where
 * receives the layout a^† o t, which maps instruction coordinates to coordinates of `a` (NULL when that composition is
 * not admissible by Sec. 3.3.2's conditions; the answer in *yes stands either way); on no, NULL.
 * Errors: those of lc_left_inverse (`a` must have a left-inverse layout); TOO_LARGE (|t| > 2^26). */
lc_status_t lc_admissible(const lc_layout_t* a, const lc_layout_t* t, int* yes, lc_layout_t** where);

/* Logical product A (x) B = (A, A* o B) (Sec. 3.5.1): mode 0 is the tile A, mode 1 repeats it over the
 * grid B.  Errors of lc_complement and lc_composition. */
lc_status_t lc_logical_product(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out);
/* The logical product with like modes paired (Sec. 3.5.1, related products); needs rank(a) == rank(b).
 * blocked: ((A_0,B'_0),(A_1,B'_1),...); raked: ((B'_0,A_0),(B'_1,A_1),...) with B' = A* o B. */
lc_status_t lc_blocked_product(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out);
lc_status_t lc_raked_product(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out);

/* Logical divide A (/) B = A o (B, B*_{|A|}) (Sec. 3.5.2): rank 2, mode 0 = A o B, mode 1 = the rest. */
lc_status_t lc_logical_divide(const lc_layout_t* a, const lc_layout_t* b, lc_layout_t** out);
/* Logical divide applied to the top-level modes with a tiler (Sec. 3.5.2, related divides). */
lc_status_t lc_logical_divide_bymode(const lc_layout_t* a, const lc_layout_t* tiler, lc_layout_t** out);
/* By-mode logical divide, then like modes zipped: ((tile_0, tile_1, ...), (rest_0, rest_1, ..., untouched modes)). */
lc_status_t lc_zipped_divide(const lc_layout_t* a, const lc_layout_t* tiler, lc_layout_t** out);

/* Largest K such that the first K offsets of both layouts belong to the same coordinates: the extent of the
 * stride-1 head of coalesce(a o right_inverse(b)) (Sec. 3.4.2).  Requires |a| == |b|. */
lc_status_t lc_max_common_vector(const lc_layout_t* a, const lc_layout_t* b, int64_t* K);

/* ---------------------------------------------------------------------------------------------
 * Layouts with integer-semimodule strides (Sec. 2.3.2, Fig. layouts2).  Host objects like lc_layout_t.
 * Text form as the paper prints them: integers, scaled basis elements "e0", "6e1" of Z^(*,..,*) (the
 * layout then yields a coordinate with one component per axis), or XOR elements "f5" of (Z, XOR, *)
 * (a swizzled offset), e.g. "(4,(4,2)):(e1,(e0,6e1))", "(8,8):(f1,f9)".  The inner product is taken
 * in the semimodule: c * (a e_i) = (c a) e_i added per component, c * f_d = f_(c d) added by XOR.
 * One kind of stride per layout (zeros aside); at most 16 axes.
 * lc_slayout_kind: 0 integer, 1 coordinate, 2 XOR.  lc_slayout_eval writes lc_slayout_codomain_rank()
 * values to out (cap = room in out); the extended domain applies as for lc_layout_eval.
 * lc_slayout_composition: A o B for an integer layout B (Sec. 3.3 "Reductive case: Coordinate",
 * Table TVLayoutExamples rows Swizzled and Coordinate); errors as lc_composition.  With XOR strides the
 * modes of B that walk one mode of A are added as integers before A scales them, which is their XOR only while no two
 * of them can set the same bit (true for the paper's example): otherwise no layout with XOR strides equals A(B(c)) and
 * the call answers NOT_SEGREGATED; TOO_LARGE when a mode is too long to decide that (more than 2^24 positions).
 * lc_slayout_coalesce: Sec. 3.2 in the semimodule (XOR modes never merge).
 * lc_slayout_right_inverse: coordinate layouts only (Table rinv, rows with e_i strides): the integer
 * layout R on the largest box of coordinates starting at 0 with A(R(c)) = c; INVALID_ARG otherwise.
 * Errors of parse: PARSE, NOT_CONGRUENT, BAD_EXTENT, INVALID_ARG (mixed kinds, size overflow). */
lc_status_t lc_slayout_parse(const char* text, lc_slayout_t** out);
void lc_slayout_destroy(lc_slayout_t* layout);
lc_status_t lc_slayout_to_string(const lc_slayout_t* layout, char* buf, size_t cap, size_t* needed);
int lc_slayout_kind(const lc_slayout_t* layout);
int lc_slayout_codomain_rank(const lc_slayout_t* layout);
int64_t lc_slayout_size(const lc_slayout_t* layout);
lc_status_t lc_slayout_eval(const lc_slayout_t* layout, int64_t integral_coord, int64_t* out, int cap);
lc_status_t lc_slayout_composition(const lc_slayout_t* a, const lc_layout_t* b, lc_slayout_t** out);
lc_status_t lc_slayout_coalesce(const lc_slayout_t* a, lc_slayout_t** out);
lc_status_t lc_slayout_right_inverse(const lc_slayout_t* a, lc_layout_t** out);
/* lc_slayout_xor_right_inverse: layouts with XOR strides (Table rinv, last row, which only says that one can be defined; this
 * reading): *out = (2,...,2):(f_x0, f_x1, ...), x_b the smallest integral coordinate of a whose offset is 2^b, up to the first power
 * of two a does not reach (nothing: 1:0); then a(out(k)) = k for every k < size(out).  Host work only.  a must be additive over XOR
 * of integral coordinates -- extents powers of two, no carry among a stride's multiples inside its mode -- else LC_ERR_INVALID_ARG;
 * the caller destroys *out. */
lc_status_t lc_slayout_xor_right_inverse(const lc_slayout_t* a, lc_slayout_t** out);

/* ---------------------------------------------------------------------------------------------
 * COPY (Sec. 2.6.1): dst(i) = src(i) for i in [0, size(dst)), executed on the GPU.
 * The plan coalesces both layouts, refines them to a common shape, permutes the iteration order
 * consistently on both sides (Sec. 3.4.2), picks the common vector width and tiles the copy with
 * zipped_divide (Sec. 3.5.2); plan creation is pure host work and touches no device.
 * ------------------------------------------------------------------------------------------- */

/* src_align_bytes / dst_align_bytes: alignment the caller guarantees for the device pointers that
 * will be passed to lc_plan_execute (a power of two; 256 for fresh allocations).  Errors: SIZE_MISMATCH,
 * UNSUPPORTED_DTYPE, TOO_LARGE.
 * Destination modes of stride 0 do not count as aliasing: the loop of Sec. 2.6.1 runs i upwards, so the
 * coordinate with those modes at their last position is the one written last, and the plan copies exactly
 * that slice of the source (Sec. 2.5.1; lc_plan_describe reports overwritten_modes and src_offset).  Any
 * other overlap in dst (strides that make distinct coordinates meet), and a dst of more than 2^22 elements whose
 * strides are not nested (each at least the extent of the modes below it; its injectivity is not proved cheaply),
 * gives a plan of class "last-writer", which needs a workspace: see lc_plan_execute_workspace. */
lc_status_t lc_plan_create(const lc_layout_t* src, const lc_layout_t* dst, lc_dtype_t dt,
                           unsigned src_align_bytes, unsigned dst_align_bytes, lc_plan_t** out);
/* One-line description: kernel class, vector width, joint modes, tile, grid, LDS bytes, swizzle. */
lc_status_t lc_plan_describe(const lc_plan_t* plan, char* buf, size_t cap, size_t* needed);
/* Enqueue the copy on `hip_stream`.  Asynchronous; allocates nothing, copies nothing, synchronises nothing (it may be
 * recorded into a HIP graph).  Errors: MISALIGNED, HIP.
 * Long transposing copies hand their tiles, and contiguous copies of 2 GiB or more their chunks, out through a block of
 * counters in device memory of the library's own code object, one block per stream (the library's launches on a stream
 * run in stream order, which is what keeps a block to one kernel at a time); launches on more than 64 streams of a
 * device, launches under graph capture, launches on the per-thread default stream handle (hipStreamPerThread: one handle
 * value, a different stream in every host thread) and launches on a stream of another device than the current one use a
 * fixed order instead.  A stream that is destroyed with such a copy still queued, and whose handle value the runtime then
 * gives to a new stream, would share its block with it: synchronise before destroying the stream. */
lc_status_t lc_plan_execute(const lc_plan_t* plan, const void* src, void* dst, void* hip_stream);
/* Scatter with repeated destination offsets (Table copy, Sec. 2.6.1): the loop runs i upwards, so an offset that several
 * integral coordinates reach keeps the value of the largest of them.  A destination that aliases in another way than
 * through modes of stride 0, or whose distinctness cannot be shown on the host (more than 2^22 elements with strides that
 * do not nest), plans as class "last-writer": a first pass records, per destination offset, the largest coordinate that
 * reaches it (atomic maximum into one 32-bit word per element of cosize(dst)), a second pass lets only those coordinates
 * write.  Such a plan needs lc_plan_workspace_bytes(plan) bytes of scratch device memory (0 for every other plan), which
 * the caller owns and passes to lc_plan_execute_workspace (4-byte aligned; contents before and after the call are
 * meaningless; two executions that overlap in time need two workspaces).  lc_plan_execute and lc_copy return
 * NEEDS_WORKSPACE for such a plan; lc_plan_execute_workspace runs every other plan as lc_plan_execute does and ignores the
 * workspace.  Errors: WORKSPACE_TOO_SMALL (NULL, misaligned or short), MISALIGNED, HIP. */
int64_t lc_plan_workspace_bytes(const lc_plan_t* plan);
lc_status_t lc_plan_execute_workspace(const lc_plan_t* plan, const void* src, void* dst, void* workspace, size_t workspace_bytes,
                                      void* hip_stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it): lc_plan_execute_workspace with the scratch memory taken from a static array in device memory of the
 * library's own code object, LC_STATIC_SCRATCH_BYTES (8 MiB) per GPU, which every GPU the library runs on holds until the
 * process ends.  Calls nothing that allocates.  A plan that needs more (lc_plan_workspace_bytes(plan) >
 * lc_static_scratch_bytes()) is refused with SCRATCH_LIMIT; a plan that needs no scratch runs as lc_plan_execute does.
 * All calls on a GPU share that GPU's array, whatever the stream, and the array keeps what the last call left in it
 * (each call clears the part it uses with a kernel of its own, so stale contents do no harm): two calls that overlap in
 * time on one GPU race on it; calls on one stream, or ordered by events, do not.  The array used is the current
 * device's (hipGetDevice), which must be the device of `hip_stream`. */
#define LC_STATIC_SCRATCH_BYTES (8u << 20)
size_t lc_static_scratch_bytes(void);
lc_status_t lc_plan_execute_static(const lc_plan_t* plan, const void* src, void* dst, void* hip_stream);
void lc_plan_destroy(lc_plan_t* plan);

/* lc_plan_create (alignment taken from the two pointers) + lc_plan_execute + lc_plan_destroy.  The library keeps the
 * plans of recent calls (up to 256, keyed by both layouts, dtype, the pointers' alignment and the LC_TUNE_* settings),
 * so a repeated call only pays for the launch; thread-safe.  lc_gemm does the same. */
lc_status_t lc_copy(const void* src, const lc_layout_t* src_layout, void* dst, const lc_layout_t* dst_layout,
                    lc_dtype_t dt, void* hip_stream);

/* Bytes the plan moves per execution: elements * element width, once read and once written
 * (a stride-0 source mode re-reads count once). */
int64_t lc_plan_algorithmic_bytes(const lc_plan_t* plan);

/* Times `iters` back-to-back executions of the plan on `hip_stream` with HIP events recorded on that
 * same stream, after `warmup` untimed ones; returns the mean milliseconds per execution in *ms_per_iter.
 * Synchronises the stream (the only call here that does).  `srcs`/`dsts` are host arrays of `n_buffers`
 * device pointers used round-robin, so that successive executions touch different memory. */
lc_status_t lc_plan_time(const lc_plan_t* plan, const void* const* srcs, void* const* dsts, int n_buffers,
                         int warmup, int iters, void* hip_stream, float* ms_per_iter);
/* The same executions with a HIP event between every two of them: ms_each (host array of `iters` floats, iters <= 4096)
 * receives, per execution, the time between the events around it: a median and a minimum beside lc_plan_time's mean.
 * An event between two short kernels delays the second by about a microsecond, so for kernels of a few microseconds
 * these figures lie above lc_plan_time's.  Errors: INVALID_ARG, HIP, and those of lc_plan_execute. */
lc_status_t lc_plan_time_each(const lc_plan_t* plan, const void* const* srcs, void* const* dsts, int n_buffers,
                              int warmup, int iters, void* hip_stream, float* ms_each);

/* ---------------------------------------------------------------------------------------------
 * GEMM (Sec. 2.6.2): C(m,n) += A(m,k) * B(n,k) for every m < M, n < N, k < K, executed on the GPU's
 * matrix cores.  Each tensor is a device pointer and a layout of rank 2 whose modes may be multi-modes
 * (Table gemm: BLAS N/T variants, BLIS strides, GETT foldings, im2col views):
 *     A over (M,K), B over (N,K), C over (M,N)
 * with M = size<0>(A) = size<0>(C), N = size<0>(B) = size<1>(C), K = size<1>(A) = size<1>(B) (the
 * preconditions of Sec. 2.6.2; SIZE_MISMATCH otherwise, INVALID_ARG for a layout that is not rank 2).
 * Batched form (Sec. 1, the canonical contraction C(m,n,l) += A(m,k,l) * B(n,k,l)): all three layouts of rank 3,
 * A over (M,K,L), B over (N,K,L), C over (M,N,L), the third modes of equal size L <= 65535 (a stride-0 batch
 * mode shares one operand between all batch entries); the flop count is then 2 M N K L.
 * A and B hold bf16 or fp16 elements (`ab_dtype` = LC_BF16 / LC_F16, the same for both), C holds fp32;
 * products are exact and sums are accumulated in fp32, in an order that differs from the loop nest's
 * (the result is within K * 2^-23 * sum_k |A(m,k) B(n,k)| of the exactly accumulated value).
 * Strides count elements of the respective tensor.  The caller guarantees cosize(layout) elements
 * behind each pointer; A and B may alias each other, C may alias neither.
 * The planner coalesces every mode (Sec. 3.2), loads an operand with 16-byte vectors along whichever
 * of its modes leads with a contiguous run of 8 elements (along k: straight into LDS; along m / n:
 * through a register transpose), element by element otherwise, and exchanges the roles of A and B
 * when C is contiguous along n rather than m.  Errors: DST_ALIASES (two coordinates of C share an
 * offset), UNSUPPORTED_DTYPE, TOO_LARGE (a cosize or extent of 2^31 or more, more than 4 leaves left
 * in a coalesced mode), MISALIGNED (execute: a pointer less aligned than the plan was created for), HIP.
 * ------------------------------------------------------------------------------------------- */
lc_status_t lc_gemm_plan_create(const lc_layout_t* a, const lc_layout_t* b, const lc_layout_t* c, lc_dtype_t ab_dtype,
                                unsigned a_align_bytes, unsigned b_align_bytes, unsigned c_align_bytes, lc_gemm_plan_t** out);
/* One line: tile, grid, how each operand is loaded, the coalesced modes. */
lc_status_t lc_gemm_plan_describe(const lc_gemm_plan_t* plan, char* buf, size_t cap, size_t* needed);
/* Enqueue on `hip_stream`; asynchronous; a, b, c are device pointers. */
lc_status_t lc_gemm_plan_execute(const lc_gemm_plan_t* plan, const void* a, const void* b, void* c, void* hip_stream);
void lc_gemm_plan_destroy(lc_gemm_plan_t* plan);
/* lc_gemm_plan_create (alignment taken from the pointers) + lc_gemm_plan_execute. */
lc_status_t lc_gemm(const void* a, const lc_layout_t* a_layout, const void* b, const lc_layout_t* b_layout, void* c,
                    const lc_layout_t* c_layout, lc_dtype_t ab_dtype, void* hip_stream);
int64_t lc_gemm_plan_flops(const lc_gemm_plan_t* plan); /* 2 M N K (L) */
/* Mean milliseconds of `iters` back-to-back executions after `warmup` untimed ones, by HIP events on
 * `hip_stream`; synchronises the stream.  C accumulates across the executions. */
lc_status_t lc_gemm_plan_time(const lc_gemm_plan_t* plan, const void* a, const void* b, void* c, int warmup, int iters,
                              void* hip_stream, float* ms_per_iter);
/* Thread-value layouts (Sec. 3.3.4, Table TVLayoutExamples) of the fragments of the matrix instruction the
 * GEMM kernel uses, v_mfma_f32_32x32x16 (bf16 / f16): (lane, value) -> integral coordinate in the fragment's
 * tile, column-major.  which = 0: A, (64,8) -> m + 32 k of the (32,16) tile; 1: B, (64,8) -> n + 32 k;
 * 2: C, (64,16) -> m + 32 n of the (32,32) tile. */
lc_status_t lc_mfma_fragment_layout(int which, lc_layout_t** out);

#ifdef __cplusplus
}
#endif
#endif /* LAYOUTCOPY_H_ */
