/* tcx.h -- C interface of libtcx: general binary tensor contraction on one AMD MI355X.
 *
 *     D := alpha * opA(A) * opB(B) + beta * opC(C)          (paper, Eq. binary_contraction)
 *
 * A, B, C, D are dense tensors in a general strided layout (glossary, "Strided layout":
 * address = base + sum_k i_k * s_k).  Every mode carries an integer label.  A label that
 * occurs in A and B only is contracted (summed, set P); in A and D only, or in B and D
 * only, it is free (F_A, F_B); in A, B and D it is a Hadamard / batch label (H)
 * (Secs. "Case 1", "Case 2", Eqs. case1, case2).  A label repeated inside one tensor
 * addresses a diagonal (Sec. "Case 3", Note 6).  A label that occurs in A only, or in B
 * only, is summed inside that tensor before the product (Sec. "Case 4": the operand is
 * reduced by a kernel of its own into workspace memory, TCX_KEY_WORKSPACE_BYTES); a label
 * that occurs in D (and C) only repeats the product for each of its values (Sec. "Case 5").
 * The standard does not require the last two (Note 7); this library computes them.
 *
 * Object model (Sec. "Interface Components"): a library handle, an executor (a HIP
 * stream), tensor descriptors ("tensor info": rank, extents, strides, dtype -- no data
 * pointer), a product plan built from four descriptors, their labels, the element-wise
 * ops and a precision, an execute call that takes only data pointers and scalars, an
 * optional status object, and integer error codes with a text explanation
 * (Sec. "Error Handling").  All handles are opaque integers; 0 is "no object".
 *
 * Conventions
 *  - Every function returns a tcx_error_t; 0 is success.  Outputs come back through
 *    pointers; where noted an output pointer may be NULL to skip it.
 *  - Ownership: the library owns an object from create to destroy.  destroy takes the
 *    handle by pointer and sets it to 0.  The library never owns tensor data.  A product
 *    copies what it needs from its tensor infos, which may be destroyed right after.
 *  - Strides are in ELEMENTS (not bytes), signed.  A data pointer addresses the element
 *    whose indices are all zero.  Zero strides are legal in A and B (broadcast), not in D.
 *  - Data pointers passed to tcx_execute_product are DEVICE pointers on the handle's GPU.
 *    alpha and beta are HOST pointers to one element of D's dtype (two doubles for
 *    TCX_C128, two floats for TCX_C64) and are read before the call returns.
 *  - beta == 0: C is never read and may be NULL; D is overwritten.  alpha == 0: A and B
 *    are never read.  C may be the same pointer as D (in place); any other overlap of
 *    D with A, B or C is undefined.  Buffer elements of D that (extents, strides) do not
 *    address are left bit-unchanged.
 *  - tcx_execute_product enqueues work on the executor's stream and returns; argument
 *    errors are reported synchronously, before anything is enqueued.
 *  - Objects are immutable after creation (tcx_product_set and the executor's keys aside), so
 *    one product may be executed from several threads and on several executors at once.  A
 *    product whose plan cuts the contracted range into parts (TCX_KEY_SPLIT_K > 1) writes
 *    partial sums to a device workspace that belongs to the EXECUTOR: work on one stream runs in
 *    order, so executions through one executor share it safely (calls from several host threads
 *    through one executor are enqueued one after the other), and executions through different
 *    executors use different buffers.  The workspace grows on demand inside tcx_execute_product
 *    (the only device allocation an execution can make; TCX_KEY_WORKSPACE_BYTES on the product
 *    says how much it needs, the same key set on an executor reserves it ahead of time); if that
 *    allocation fails the product runs unsplit.
 */
#ifndef TCX_H
#define TCX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tcx_error_t;
typedef intptr_t tcx_handle_t;
typedef intptr_t tcx_executor_t;
typedef intptr_t tcx_tensor_info_t;
typedef intptr_t tcx_product_t;
typedef intptr_t tcx_status_t;

/* Element types (Sec. "The Reference Implementation": real and complex, 64 and 32 bit, and real
 * 16 bit; the four tensors of a product share one).  Complex elements are (re, im) pairs of their
 * real type.  TCX_F16 is IEEE 754 binary16 and TCX_BF16 is bfloat16 (the upper half of a binary32):
 * the tensors hold 16-bit elements, products and sums are formed in 32-bit reals
 * (TCX_PREC_DEFAULT) or 64-bit reals (TCX_PREC_F64), D is rounded to 16 bits once, on the store
 * (to nearest, ties to even), and alpha and beta are passed as floats. */
typedef enum { TCX_F32 = 0, TCX_F64 = 1, TCX_C64 = 2, TCX_C128 = 3, TCX_F16 = 4, TCX_BF16 = 5 } tcx_dtype_t;
typedef enum { TCX_OP_IDENTITY = 0, TCX_OP_CONJ = 1 } tcx_op_t;          /* conj of a real type is the identity */
/* The plan's "desired computational precision" (Sec. "Tensor Operation Descriptors").
 *   TCX_PREC_DEFAULT  products and sums in the dtype's own real type (fp32 means fp32 MFMA; 16-bit
 *                     tensors: 32-bit reals);
 *   TCX_PREC_F64      products and sums in 64-bit reals whatever the storage type: 32-bit elements
 *                     are widened as they are read, alpha, beta and C are applied in 64 bits and D
 *                     is rounded once, on the store.  The same as the default for 64-bit dtypes. */
typedef enum { TCX_PREC_DEFAULT = 0, TCX_PREC_F64 = 1 } tcx_prec_t;

enum {
    TCX_SUCCESS = 0,
    TCX_ERR_NULL_ARG = 1,            /* a required pointer argument is NULL */
    TCX_ERR_INVALID_HANDLE = 2,      /* handle is 0, destroyed, or of another object type */
    TCX_ERR_BAD_DTYPE = 3,
    TCX_ERR_BAD_NMODE = 4,           /* number of modes < 0 or > TCX_MAX_MODES */
    TCX_ERR_BAD_EXTENT = 5,          /* an extent is <= 0 (Sec. Preliminaries: extents are positive) */
    TCX_ERR_EXTENT_MISMATCH = 6,     /* one label, two extents (Sec. Preliminaries; appendix test 26) */
    TCX_ERR_CD_MISMATCH = 7,         /* C is not described exactly like D (Note 5; appendix test 27) */
    TCX_ERR_D_ALIASING = 8,          /* two index tuples of D share an address (appendix test 28) */
    TCX_ERR_ISOLATED_INDEX = 9,      /* tcx_create_unary: A and B do not carry the same set of labels (contractions reduce or broadcast such labels, Secs. "Case 4", "Case 5") */
    TCX_ERR_DTYPE_MIX = 10,          /* the four tensors do not share one dtype */
    TCX_ERR_UNSUPPORTED_OP = 11,     /* op value unknown, or opD != identity */
    TCX_ERR_UNSUPPORTED_PRECISION = 12,
    TCX_ERR_ALLOC = 13,              /* host or device allocation failed */
    TCX_ERR_LAUNCH = 14,             /* the HIP runtime refused a launch or copy; see the status object */
    TCX_ERR_NO_DEVICE = 15,          /* the handle was created without a usable gfx950 GPU (plans only) */
    TCX_ERR_TOO_LARGE = 16,          /* an offset or an index range exceeds what the kernels address */
    TCX_ERR_BAD_KEY = 17,            /* unknown key in tcx_status_get / tcx_product_get / tcx_attr_*, or a free-form key that holds no value */
    TCX_ERR_BUFFER_TOO_SMALL = 18,   /* *nbytes is smaller than the value; *nbytes is set to the need */
    TCX_ERR_PLAN_REFUSED = 19,       /* tcx_product_set: this plan cannot take the requested path, tile shape or split */
    TCX_ERR_SCRATCH_TOO_SMALL = 20   /* the product needs more scratch memory than the library's fixed buffer holds */
};

#define TCX_MAX_MODES 32

/* ---- library handle (Sec. "The Library Handle") -------------------------------------
 * Binds to the current HIP device.  If no gfx950 device is usable the handle is still
 * created in plan-only state: descriptors and products can be built and inspected,
 * tcx_execute_product returns TCX_ERR_NO_DEVICE.  `out` must not be NULL. */
tcx_error_t tcx_create_handle(tcx_handle_t* out);
tcx_error_t tcx_destroy_handle(tcx_handle_t* handle);
/* 1 if the handle can execute (a gfx950 device is bound), else 0. out must not be NULL. */
tcx_error_t tcx_handle_has_device(tcx_handle_t handle, int32_t* out);

/* ---- executor (Sec. "Executors") ----------------------------------------------------
 * Wraps a hipStream_t owned by the caller (passed as void*; NULL is the default stream).
 * The stream must stay alive while the executor is in use. */
tcx_error_t tcx_create_executor(tcx_handle_t handle, void* hip_stream, tcx_executor_t* out);
tcx_error_t tcx_destroy_executor(tcx_executor_t* executor);

/* ---- tensor descriptor (Sec. "Tensor Descriptors") ----------------------------------
 * extents[nmode], strides[nmode]: host arrays, copied.  nmode may be 0 (a scalar; the
 * array pointers may then be NULL). */
tcx_error_t tcx_create_tensor_info(tcx_handle_t handle, tcx_dtype_t dtype, int32_t nmode,
                                   const int64_t* extents, const int64_t* strides, tcx_tensor_info_t* out);
tcx_error_t tcx_destroy_tensor_info(tcx_tensor_info_t* info);
/* Any output pointer may be NULL; extents/strides must hold nmode entries. */
tcx_error_t tcx_tensor_info_get(tcx_tensor_info_t info, tcx_dtype_t* dtype, int32_t* nmode,
                                int64_t* extents, int64_t* strides);

/* ---- product plan (Sec. "Tensor Operation Descriptors") -----------------------------
 * labelsX[nmode of X]: host arrays of integer labels, copied.  Validation and the index
 * analysis (classification into H / F_A / F_B / P, merging of repeated labels, fusion of
 * contiguous modes, choice of kernel path and tile plan) happen here, once, so that their
 * cost is amortised over executions.  On a handle with a device this also uploads the
 * plan's offset tables (synchronous, default stream).  C must be laid out like D (Note 5): the
 * same set of labels and, per distinct label, D's extent and D's stride (the strides of a
 * repeated label summed); the order in which C's modes are listed is free.  opD must be
 * TCX_OP_IDENTITY. */
tcx_error_t tcx_create_product(tcx_handle_t handle,
                               tcx_op_t opA, tcx_tensor_info_t A, const int64_t* labelsA,
                               tcx_op_t opB, tcx_tensor_info_t B, const int64_t* labelsB,
                               tcx_op_t opC, tcx_tensor_info_t C, const int64_t* labelsC,
                               tcx_op_t opD, tcx_tensor_info_t D, const int64_t* labelsD,
                               tcx_prec_t precision, tcx_product_t* out);
tcx_error_t tcx_destroy_product(tcx_product_t* product);

/* Keys of tcx_product_get / tcx_status_get.  Values are int64_t unless noted. */
enum {
    TCX_KEY_PATH = 1,          /* tcx_path_t chosen by the analyser */
    TCX_KEY_SIZE_H = 2,        /* product of the extents of the Hadamard labels */
    TCX_KEY_SIZE_M = 3,        /* ... of the free labels of A */
    TCX_KEY_SIZE_N = 4,        /* ... of the free labels of B */
    TCX_KEY_SIZE_K = 5,        /* ... of the contracted labels */
    TCX_KEY_NMODES_H = 6,      /* number of modes per group after merging and fusion */
    TCX_KEY_NMODES_M = 7,
    TCX_KEY_NMODES_N = 8,
    TCX_KEY_NMODES_K = 9,
    TCX_KEY_TILE_M = 10,       /* macro-tile extents of the chosen kernel (0 if not tiled) */
    TCX_KEY_TILE_N = 11,
    TCX_KEY_TILE_K = 12,
    TCX_KEY_GRID = 13,         /* number of workgroups launched */
    TCX_KEY_BLOCK = 14,        /* threads per workgroup */
    TCX_KEY_A_K_FASTEST = 15,  /* 1 if A's smallest stride belongs to a contracted mode */
    TCX_KEY_B_K_FASTEST = 16,
    TCX_KEY_D_N_FASTEST = 17,  /* 1 if D's smallest stride belongs to a free mode of B */
    TCX_KEY_VARIANT = 18,      /* index of the kernel instantiation inside the path */
    TCX_KEY_HIP_ERROR = 19,    /* status only: last hipError_t seen by the execute call */
    TCX_KEY_MODES_M = 20,      /* int64_t[4 * nmodes]: (extent, strideA, strideB, strideD) per fused mode, fastest first */
    TCX_KEY_MODES_N = 21,
    TCX_KEY_MODES_K = 22,
    TCX_KEY_MODES_H = 23,
    TCX_KEY_FORCE_PATH = 24,   /* tcx_product_set only: force a tcx_path_t (testing, tuning) */
    TCX_KEY_SPLIT_K = 25,      /* tiled path: number of parts the contracted range is cut into (1 = unsplit) */
    TCX_KEY_LAUNCHES = 26,     /* read-only: kernel launches one execution enqueues (rounds of a long-tile product; +1 for the split-K reduction; +1 per operand reduced over isolated labels) */
    TCX_KEY_GATHER_WIDTH = 27, /* read-only: elements one gather load of the tiled kernel brings (2: neighbouring pairs of 8-byte elements; a status reports what the execution used, which also depends on the operand pointers being 16-byte aligned) */
    TCX_KEY_TABLE_ENTRIES = 28,/* read-only, int64_t[3]: entries of the plan's offset tables over M, N, K including padding (0 before the tiled path was prepared) */
    TCX_KEY_WORKSPACE_BYTES = 29, /* product (read-only): device bytes of workspace one execution uses (split-K partial sums, operands reduced over isolated labels); executor: size of its workspace, settable to reserve at least that much */
    TCX_KEY_DEVICE = 30,       /* handle, executor (read-only): HIP device ordinal the object is bound to, -1 if none */
    TCX_KEY_NUM_CU = 31,       /* handle (read-only): compute units of the bound device */
    TCX_KEY_STREAM = 32,       /* executor: the hipStream_t as an integer; settable (the caller keeps the new stream alive) */
    TCX_KEY_PRECISION = 33,    /* product (read-only): the tcx_prec_t the plan computes in */
    TCX_KEY_PACED_LOADS = 34   /* product (read-only): 1 if the streaming plan issues a tile's loads a few at a time because the cache lines a tile reads from an operand agree in the address bits that select the L2 channel and set (all strides inside the tile multiples of 128 KB) */
};
typedef enum {
    TCX_PATH_GENERIC = 0,      /* one thread per element of D, loops over the contracted index space */
    TCX_PATH_GETT_MFMA = 1,    /* strided gather -> LDS tiles -> MFMA, fused alpha/beta scatter */
    TCX_PATH_BANDWIDTH = 2     /* streaming path for low arithmetic intensity */
} tcx_path_t;

/* Read a property of the plan.  *nbytes: in = capacity of value, out = bytes written. */
tcx_error_t tcx_product_get(tcx_product_t product, int32_t key, void* value, size_t* nbytes);
/* Override a plan decision: TCX_KEY_FORCE_PATH, or TCX_KEY_VARIANT (tiled path: index of the tile
 * shape; bandwidth path: 0 = flat tiles only, 1 = register-blocked tiles where possible), or
 * TCX_KEY_SPLIT_K.  Returns TCX_ERR_PLAN_REFUSED if the plan cannot run that way (the plan is
 * then unchanged). */
tcx_error_t tcx_product_set(tcx_product_t product, int32_t key, const void* value, size_t nbytes);

/* ---- execution (Sec. "Execution") ----------------------------------------------------
 * status may be NULL (no status object is created).  If it is not NULL, *status receives
 * a new status object (also on TCX_ERR_LAUNCH) that the caller destroys. */
tcx_error_t tcx_execute_product(tcx_product_t product, tcx_executor_t executor, tcx_status_t* status,
                                const void* alpha, const void* A, const void* B,
                                const void* beta, const void* C, void* D);

/* The same execution for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * tcx_execute_product without the status object; the call allocates nothing, on the device or on
 * the host.  Where tcx_execute_product would lease the executor's workspace (partial sums of a
 * plan with TCX_KEY_SPLIT_K > 1, TCX_KEY_WORKSPACE_BYTES of them), this call uses a fixed buffer
 * of TCX_SCRATCH_BYTES that every GPU running the library holds from load until the process ends.
 * A product that needs more returns TCX_ERR_SCRATCH_TOO_SMALL and enqueues nothing.  All calls on
 * one GPU share that buffer: two of them that both need it must not overlap in time (the same
 * stream, or the caller's own ordering); the buffer keeps the last call's contents and every
 * call writes all it reads, so nothing has to be cleared. */
#define TCX_SCRATCH_BYTES (32 * 1024 * 1024)
tcx_error_t tcx_execute_product_noalloc(tcx_product_t product, tcx_executor_t executor,
                                        const void* alpha, const void* A, const void* B,
                                        const void* beta, const void* C, void* D);

/* ---- unary and binary operations (Sec. "Unary and Binary Operations") ----------------------
 * C := alpha * opA(A) + beta * opB(B).  B and C carry the same labels and C is laid out like B
 * (as C and D of a contraction: else TCX_ERR_CD_MISMATCH); opC must be the identity.  Labels of A
 * that C lacks are summed inside A, labels of C that A lacks broadcast A's element (the paper's
 * I_A and I_B of this operation).  The plan is a tcx_product_t (same keys, tcx_destroy_product)
 * that only tcx_execute_binary accepts.  B may be the same pointer as C; beta == 0: B is never
 * read and may be NULL.
 * B := alpha * opA(A): the unary operation (scaling, copying between layouts, diagonals through
 * repeated labels).  A and B carry the same set of labels (else TCX_ERR_ISOLATED_INDEX); opB must
 * be the identity. */
tcx_error_t tcx_create_binary(tcx_handle_t handle,
                              tcx_op_t opA, tcx_tensor_info_t A, const int64_t* labelsA,
                              tcx_op_t opB, tcx_tensor_info_t B, const int64_t* labelsB,
                              tcx_op_t opC, tcx_tensor_info_t C, const int64_t* labelsC,
                              tcx_prec_t precision, tcx_product_t* out);
tcx_error_t tcx_execute_binary(tcx_product_t plan, tcx_executor_t executor, tcx_status_t* status,
                               const void* alpha, const void* A, const void* beta, const void* B, void* C);
tcx_error_t tcx_create_unary(tcx_handle_t handle,
                             tcx_op_t opA, tcx_tensor_info_t A, const int64_t* labelsA,
                             tcx_op_t opB, tcx_tensor_info_t B, const int64_t* labelsB,
                             tcx_prec_t precision, tcx_product_t* out);
tcx_error_t tcx_execute_unary(tcx_product_t plan, tcx_executor_t executor, tcx_status_t* status,
                              const void* alpha, const void* A, void* B);

/* ---- status object (Sec. "Status Objects") ------------------------------------------ */
tcx_error_t tcx_status_get(tcx_status_t status, int32_t key, void* value, size_t* nbytes);
tcx_error_t tcx_destroy_status(tcx_status_t* status);

/* ---- virtual key-value stores (Sec. "Virtual Key-Value Stores (VKVs)") -----------------
 * A mapping from integral keys to arbitrary binary values, available on every object of the
 * library through one interface, and as a bare store of its own.  `object` is any live handle,
 * executor, tensor info, product, status or bare store (else TCX_ERR_INVALID_HANDLE).
 *   keys >= TCX_KEY_USER   free-form: the library copies the nbytes bytes at `value` into the
 *                          object (value may be NULL iff nbytes == 0), returns them unchanged,
 *                          forgets them on clear and when the object is destroyed;
 *   keys <  TCX_KEY_USER   the library's own ("virtual": they read and write state kept elsewhere):
 *                          on a product the TCX_KEY_* of tcx_product_get / tcx_product_set, on a
 *                          status those of tcx_status_get; clearing TCX_KEY_FORCE_PATH,
 *                          TCX_KEY_VARIANT or TCX_KEY_SPLIT_K on a product returns the whole plan
 *                          to the analyser's own choice; on a handle TCX_KEY_DEVICE and
 *                          TCX_KEY_NUM_CU, on an executor TCX_KEY_DEVICE, TCX_KEY_STREAM and
 *                          TCX_KEY_WORKSPACE_BYTES; any other combination TCX_ERR_BAD_KEY.
 * get: *nbytes in = capacity of value, out = size of the stored value; value NULL or too small:
 * TCX_ERR_NULL_ARG / TCX_ERR_BUFFER_TOO_SMALL with *nbytes set to the need.  A key that was never
 * set (or was cleared): TCX_ERR_BAD_KEY.  The caller keeps ownership of `value` in all calls. */
#define TCX_KEY_USER 65536
typedef intptr_t tcx_attr_t;       /* a bare store */
typedef intptr_t tcx_object_t;     /* any object of the library */
tcx_error_t tcx_create_attr(tcx_handle_t handle, tcx_attr_t* out);
tcx_error_t tcx_destroy_attr(tcx_attr_t* attr);
tcx_error_t tcx_attr_set(tcx_object_t object, int32_t key, const void* value, size_t nbytes);
tcx_error_t tcx_attr_get(tcx_object_t object, int32_t key, void* value, size_t* nbytes);
tcx_error_t tcx_attr_clear(tcx_object_t object, int32_t key);

/* ---- measurement aid (not part of the contraction) -----------------------------------------
 * Enqueues ONE launch of a kernel that does a single kind of work on the executor's stream, so
 * that a benchmark can print what the chip sustains beside its specification figures:
 *   TCX_PROBE_MFMA_F64 / _F32  every wave of every compute unit issues `iters` x 16 independent
 *                              16x16x4 MFMAs back to back (buffer: at least 16 bytes, not written);
 *   TCX_PROBE_STORE            fills buffer[0, bytes) with 16-byte stores;
 *   TCX_PROBE_COPY             copies the first half of buffer[0, bytes) to the second half.
 * buffer is a device pointer, 16-byte aligned.  *work receives the flop (MFMA probes) or the bytes
 * read plus written (memory probes) of the launch; the caller times it with events. */
typedef enum { TCX_PROBE_MFMA_F64 = 0, TCX_PROBE_MFMA_F32 = 1, TCX_PROBE_STORE = 2, TCX_PROBE_COPY = 3 } tcx_probe_t;
tcx_error_t tcx_probe_launch(tcx_executor_t executor, int32_t kind, void* buffer, size_t bytes, int64_t iters, double* work);

/* ---- error handling (Sec. "Error Handling") ------------------------------------------ */
int tcx_check_success(tcx_error_t error);                                  /* 1 iff error == TCX_SUCCESS */
/* strerror analogue: writes at most maxlen bytes (NUL-terminated if maxlen > 0) and
 * returns the length the full message needs, excluding the NUL.  msg may be NULL. */
size_t tcx_explain_error(tcx_error_t error, size_t maxlen, char* msg);

#ifdef __cplusplus
}
#endif
#endif /* TCX_H */
