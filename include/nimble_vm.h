/*
 * nimble_vm.h - C ABI of a small register-based interpreter that drives the
 * dynamic-shape kernels of nimble.h from bytecode.
 *
 * The paper compiles a dynamic model to bytecode for a register VM whose
 * instructions are coarse (one per tensor-level action: allocate, invoke a
 * kernel, branch), so that the dispatch loop adds next to nothing to kernel
 * time (Section 4; instruction set in Appendix C, Table C.1).  This interpreter
 * implements the part of that instruction set which the dynamic-shape path
 * needs - shape_of, shape function, allocation from the computed shape,
 * invoke_mut, control flow - so that the LSTM token loop and a transformer
 * feed-forward block can run as programs whose tensor shapes are only known
 * when an input arrives (Appendix A's listing is the model for such a program).
 *
 * Memory: the interpreter never allocates device memory.  The caller passes a
 * device pool; AllocStorage carves blocks from it (64-byte aligned, Section
 * 3.3) and a block returns to the pool when the last register or tensor that
 * refers to it is overwritten or FreeStorage names it.  Reuse is safe because
 * every kernel of a run is enqueued on the one stream passed to nimble_vm_run.
 * Host objects (shape tensors, integers) live in ordinary host memory.
 *
 * Bytecode format: a flat array of int64 words.  One instruction is
 *     word 0      opcode (nimble_vm_opcode)
 *     word 1      n = number of operand words that follow
 *     word 2..    the n operands, in the order given per opcode below
 * (variable length: AllocTensor carries a shape, InvokePacked its registers).
 * Jump operands are RELATIVE offsets counted in instructions from the jumping
 * instruction itself (offset 1 = fall through).  Registers are numbered from 0;
 * the inputs of a run occupy registers 0..n_inputs-1.
 */
#ifndef NIMBLE_VM_H_
#define NIMBLE_VM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Opcodes: the names and meanings of Table C.1.  "r" marks a register operand. */
typedef enum nimble_vm_opcode {
  NIMBLE_OP_MOVE = 0,             /* src r, dst r                                              */
  NIMBLE_OP_RET = 1,              /* result r: ends the run, the object becomes the result     */
  NIMBLE_OP_IF = 2,               /* test r, target r, true_offset, false_offset: integers in  */
                                  /* both registers; equal -> pc += true_offset, else false    */
  NIMBLE_OP_GOTO = 3,             /* offset: pc += offset                                      */
  NIMBLE_OP_LOAD_CONST = 4,       /* index into the constant pool, dst r                       */
  NIMBLE_OP_LOAD_CONSTI = 5,      /* immediate value, dst r                                    */
  NIMBLE_OP_ALLOC_STORAGE = 6,    /* size r (integer, bytes), alignment, device (0 host,       */
                                  /* 1 GPU pool), dst r                                        */
  NIMBLE_OP_ALLOC_TENSOR = 7,     /* storage r, byte offset, dtype, rank, extents[rank], dst r */
  NIMBLE_OP_ALLOC_TENSOR_REG = 8, /* storage r, byte offset, shape r (host i64 tensor), dtype, */
                                  /* dst r                                                     */
  NIMBLE_OP_ALLOC_ADT = 9,        /* tag, count, field r[count], dst r                         */
  NIMBLE_OP_ALLOC_CLOSURE = 10,   /* not implemented here (NIMBLE_ERR_ARG at load)             */
  NIMBLE_OP_FREE_STORAGE = 11,    /* storage r: give the block back now; later use is an error */
  NIMBLE_OP_FREE_TENSOR = 12,     /* tensor r: drop the register's reference to the tensor     */
  NIMBLE_OP_INVOKE = 13,          /* not implemented here (one function per executable)        */
  NIMBLE_OP_INVOKE_CLOSURE = 14,  /* not implemented here                                      */
  NIMBLE_OP_INVOKE_PACKED = 15,   /* packed id, arity, output count, r[arity]: the last        */
                                  /* `output count` registers are outputs (invoke_mut)         */
  NIMBLE_OP_GET_FIELD = 16,       /* object r, index, dst r                                    */
  NIMBLE_OP_GET_TAG = 17,         /* object r, dst r                                           */
  NIMBLE_OP_DEVICE_COPY = 18,     /* not implemented here (inputs arrive on the GPU)           */
  NIMBLE_OP_SHAPE_OF = 19,        /* tensor r, dst r: host i64 tensor of the extents           */
  NIMBLE_OP_RESHAPE_TENSOR = 20,  /* tensor r, shape r, dst r: same data, same element count   */
  NIMBLE_OP_FATAL = 21,           /* ends the run with NIMBLE_ERR_SHAPE                        */
  NIMBLE_OP_COUNT = 22
} nimble_vm_opcode;

/* Packed functions InvokePacked can name.  Arguments are listed inputs -> outputs; "shape" is
 * a host i64 tensor, "int" an integer object, the rest are GPU tensors. */
typedef enum nimble_vm_packed {
  NIMBLE_PF_SHAPE_DENSE = 0,     /* x shape, w shape -> out shape (nimble_dense_shape)          */
  NIMBLE_PF_SHAPE_LSTM = 1,      /* x shape, h shape, c shape, w shape -> h' shape, c' shape    */
  NIMBLE_PF_SHAPE_ATTENTION = 2, /* q shape, k shape, v shape -> o shape (the two batch_matmul  */
                                 /* shape functions composed)                                   */
  NIMBLE_PF_STORAGE_BYTES = 3,   /* shape, dtype int -> int (nimble_storage_bytes)              */
  NIMBLE_PF_SHAPE_GET = 4,       /* shape, index int -> int                                     */
  NIMBLE_PF_INT_ADD = 5,         /* int, int -> int                                             */
  NIMBLE_PF_INT_LESS = 6,        /* int, int -> int (1 when a < b, else 0)                      */
  NIMBLE_PF_INDEX0 = 7,          /* tensor [T,...], t int -> tensor [...]: view of slice t, no  */
                                 /* copy (the list of per-token inputs of a sequence model)     */
  NIMBLE_PF_DENSE = 8,           /* x, w -> y                       (nimble_dense_dyn, no bias) */
  NIMBLE_PF_DENSE_BIAS = 9,      /* x, w, b -> y                                                */
  NIMBLE_PF_DENSE_BIAS_GELU = 10,/* x, w, b -> y                                                */
  NIMBLE_PF_LSTM_GATES = 11,     /* x, h, w, b, c -> c', h'         (nimble_lstm_gates_dyn)     */
  NIMBLE_PF_ATTENTION = 12,      /* q, k, v -> o, alpha = 1/sqrt(D) (nimble_attention_dyn)      */
  NIMBLE_PF_COUNT = 13
} nimble_vm_packed;

#define NIMBLE_I64 2 /* dtype selector of host shape tensors and integer results (VM only) */

/* A tensor as it crosses this boundary.  `data` is a device pointer for bf16/f32 tensors
 * (owned by the caller for inputs and constants; inside the caller's pool for results) and a
 * host pointer, valid until the next run or destroy, for NIMBLE_I64 results.  An integer result
 * has rank 0 and its value in shape[0]. */
typedef struct nimble_vm_tensor {
  void* data;
  int32_t dtype; /* NIMBLE_BF16, NIMBLE_F32 or NIMBLE_I64 */
  int32_t rank;  /* 0..4 */
  int64_t shape[4];
} nimble_vm_tensor;

typedef struct nimble_vm nimble_vm;

/* Load an executable: bytecode of one function, its register count and its constant pool
 * (weights; device pointers the caller keeps alive).  The code is checked once here: known
 * opcodes with the right operand counts, registers below n_registers, constant and packed ids in
 * range, every jump landing on an instruction of the function, last instruction not falling off
 * the end.  Returns NIMBLE_OK and *out, or NIMBLE_ERR_NULL / NIMBLE_ERR_ARG with a message. */
int nimble_vm_create(const int64_t* code, int64_t n_words, int64_t n_registers,
                     const nimble_vm_tensor* constants, int n_constants, nimble_vm** out);

void nimble_vm_destroy(nimble_vm* vm);

/* Run the function once.  inputs -> registers 0..n_inputs-1.  `pool` is caller-owned device
 * memory of `pool_bytes` for AllocStorage (the pool is empty at the start of every run; results
 * point into it and stay valid until the next run with the same pool).  `workspace` as in
 * nimble_dense_dyn.  At most `max_instructions` instructions execute (<= 0: 100 million); more
 * is NIMBLE_ERR_ARG, as are a type error in a register (an integer where a tensor is needed),
 * an exhausted pool (NIMBLE_ERR_WORKSPACE) and whatever a packed function returns.  The result
 * object is written to results[0..*n_results): a tensor or integer gives one entry, an ADT its
 * fields in order (nested ADTs flattened).  Kernels are enqueued on `stream`; nothing
 * synchronises.  On error the outputs of kernels already enqueued are unspecified. */
int nimble_vm_run(nimble_vm* vm, const nimble_vm_tensor* inputs, int n_inputs, void* pool,
                  uint64_t pool_bytes, void* workspace, uint64_t workspace_bytes, void* stream,
                  int64_t max_instructions, nimble_vm_tensor* results, int max_results,
                  int* n_results);

/* Host-side cost of the last run, the split the paper reports as kernel time against "others"
 * (Section 5.3, overhead study): per opcode, how many instructions ran and the host nanoseconds
 * spent in them (for InvokePacked of a GPU kernel this is dispatch + launch, not GPU time); the
 * same per packed function.  Arrays of NIMBLE_OP_COUNT and NIMBLE_PF_COUNT entries; any may be
 * NULL.  *pool_high_water = most pool bytes in use at once, *storage_allocs = AllocStorage
 * instructions on the GPU pool, *storage_reuses = how many of them were served by a returned
 * block. */
int nimble_vm_profile(const nimble_vm* vm, int64_t* op_count, int64_t* op_ns,
                      int64_t* packed_count, int64_t* packed_ns, uint64_t* pool_high_water,
                      int64_t* storage_allocs, int64_t* storage_reuses);

#ifdef __cplusplus
}
#endif
#endif /* NIMBLE_VM_H_ */
