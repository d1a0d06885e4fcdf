// Register-based bytecode interpreter over the dynamic-shape kernels (paper Section 4 and
// Appendix C).  Host code only: every tensor-level action is one coarse instruction, device
// work happens inside the nimble_*_dyn entry points that InvokePacked calls.
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstring>
#include <map>
#include <memory>
#include <vector>

#include "nimble_internal.h"
#include "nimble_vm.h"

namespace {

using nimble::fail;

constexpr int kMaxRank = 4;
constexpr int64_t kDefaultInstructionLimit = 100000000;

const char* const kOpNames[NIMBLE_OP_COUNT] = {
    "Move", "Ret", "If", "Goto", "LoadConst", "LoadConsti", "AllocStorage", "AllocTensor",
    "AllocTensorReg", "AllocADT", "AllocClosure", "FreeStorage", "FreeTensor", "Invoke",
    "InvokeClosure", "InvokePacked", "GetField", "GetTag", "DeviceCopy", "ShapeOf",
    "ReshapeTensor", "Fatal"};

// Operand words of the fixed-length opcodes; -1 = variable (checked separately), -2 = refused.
const int kOperands[NIMBLE_OP_COUNT] = {2, 1, 4, 1, 2, 2, 4, -1, 5, -1, -2, 1, 1, -2, -2, -1,
                                        3, 2, -2, 2, 3, 0};

struct PackedInfo {
  const char* name;
  int inputs, outputs;
};
const PackedInfo kPacked[NIMBLE_PF_COUNT] = {
    {"shape_dense", 2, 1}, {"shape_lstm", 4, 2},    {"shape_attention", 3, 1},
    {"storage_bytes", 2, 1}, {"shape_get", 2, 1},   {"int_add", 2, 1},
    {"int_less", 2, 1},    {"index0", 2, 1},        {"dense", 2, 1},
    {"dense_bias", 3, 1},  {"dense_bias_gelu", 3, 1}, {"lstm_gates", 5, 2},
    {"attention", 3, 1}};

int64_t dtype_size(int dtype) {
  switch (dtype) {
    case NIMBLE_BF16: return 2;
    case NIMBLE_F32: return 4;
    case NIMBLE_I64: return 8;
    default: return 0;
  }
}

// The caller's device pool: bump allocation plus a free list of returned blocks, whole blocks
// only (a sequence model asks for the same sizes every token, so exact reuse is the common case).
struct Pool {
  char* base = nullptr;
  uint64_t bytes = 0, top = 0, in_use = 0, high_water = 0;
  uint64_t generation = 0;
  int64_t allocs = 0, reuses = 0;
  std::multimap<uint64_t, uint64_t> free_blocks;  // size -> offset

  void reset(void* b, uint64_t n) {
    base = static_cast<char*>(b);
    bytes = n;
    top = in_use = high_water = 0;
    allocs = reuses = 0;
    free_blocks.clear();
    ++generation;
  }
  bool take(uint64_t size, uint64_t align, uint64_t* offset, uint64_t* got) {
    ++allocs;
    // accept a returned block of up to twice the request that is aligned as asked, else grow
    for (auto it = free_blocks.lower_bound(size); it != free_blocks.end() && it->first <= 2 * size; ++it) {
      if (it->second % align) continue;
      *offset = it->second;
      *got = it->first;
      free_blocks.erase(it);
      ++reuses;
      in_use += *got;
      if (in_use > high_water) high_water = in_use;
      return true;
    }
    const uint64_t start = (top + align - 1) / align * align;
    if (start > bytes || size > bytes - start) return false;
    *offset = start;
    *got = size;
    top = start + size;
    in_use += size;
    if (in_use > high_water) high_water = in_use;
    return true;
  }
  void give(uint64_t offset, uint64_t size) {
    free_blocks.emplace(size, offset);
    in_use -= size;
  }
};

struct Storage {
  bool device = false;
  bool freed = false;
  uint64_t offset = 0, bytes = 0;
  Pool* pool = nullptr;
  uint64_t generation = 0;
  std::vector<int64_t> host;  // host storage, 8-byte words
  void release() {
    if (device && !freed && pool && pool->generation == generation) pool->give(offset, bytes);
    freed = true;
  }
  ~Storage() { release(); }
};

struct Object;
using Ref = std::shared_ptr<Object>;

struct Object {
  enum Kind { kInt, kStorage, kTensor, kAdt } kind = kInt;
  int64_t ival = 0;                  // kInt; tag of kAdt
  std::shared_ptr<Storage> storage;  // kStorage; backing block of a kTensor (null: caller-owned)
  void* data = nullptr;              // kTensor
  int dtype = 0, rank = 0;
  int64_t shape[kMaxRank] = {0, 0, 0, 0};
  bool on_host = false;
  std::vector<Ref> fields;  // kAdt
};

Ref make_int(int64_t v) {
  auto o = std::make_shared<Object>();
  o->kind = Object::kInt;
  o->ival = v;
  return o;
}

Ref make_host_shape(const int64_t* values, int n) {
  auto st = std::make_shared<Storage>();
  st->host.assign(values, values + n);
  st->bytes = 8u * n;
  auto o = std::make_shared<Object>();
  o->kind = Object::kTensor;
  o->storage = st;
  o->data = st->host.data();
  o->dtype = NIMBLE_I64;
  o->rank = 1;
  o->shape[0] = n;
  o->on_host = true;
  return o;
}

int64_t elements(const Object& t) {
  int64_t n = 1;
  for (int i = 0; i < t.rank; ++i) n *= t.shape[i];
  return n;
}

struct Instr {
  int op;
  std::vector<int64_t> a;
};

}  // namespace

struct nimble_vm {
  std::vector<Instr> code;
  int64_t n_registers = 0;
  std::vector<Ref> constants;
  std::vector<Ref> regs;
  Ref result;
  Pool pool;
  int64_t op_count[NIMBLE_OP_COUNT] = {0}, op_ns[NIMBLE_OP_COUNT] = {0};
  int64_t pf_count[NIMBLE_PF_COUNT] = {0}, pf_ns[NIMBLE_PF_COUNT] = {0};
  void* workspace = nullptr;
  uint64_t workspace_bytes = 0;
  void* stream = nullptr;
  // objects give their blocks back to `pool` when they die: drop them before the pool goes
  ~nimble_vm() {
    result.reset();
    regs.clear();
  }
};

namespace {

Ref from_boundary(const nimble_vm_tensor& t, int* err, const char* what, int index) {
  if (t.rank < 0 || t.rank > kMaxRank) {
    *err = fail(NIMBLE_ERR_RANK, "%s %d: rank %d outside 0..%d", what, index, t.rank, kMaxRank);
    return nullptr;
  }
  if (t.dtype != NIMBLE_BF16 && t.dtype != NIMBLE_F32) {
    *err = fail(NIMBLE_ERR_DTYPE, "%s %d: dtype %d is neither bf16 nor f32", what, index, t.dtype);
    return nullptr;
  }
  auto o = std::make_shared<Object>();
  o->kind = Object::kTensor;
  o->data = t.data;
  o->dtype = t.dtype;
  o->rank = t.rank;
  for (int i = 0; i < t.rank; ++i) {
    if (t.shape[i] < 0) {
      *err = fail(NIMBLE_ERR_ARG, "%s %d: negative extent", what, index);
      return nullptr;
    }
    o->shape[i] = t.shape[i];
  }
  if (t.data == nullptr && elements(*o) != 0) {
    *err = fail(NIMBLE_ERR_NULL, "%s %d: null data pointer", what, index);
    return nullptr;
  }
  return o;
}

// ---- typed register access: a wrong kind is the VM's run-time type error
struct Frame {
  nimble_vm* vm;
  int64_t pc;
  int err = 0;

  const Ref& reg(int64_t r) { return vm->regs[r]; }
  int bad(int64_t r, const char* want) {
    err = fail(NIMBLE_ERR_ARG, "pc %lld: register %lld does not hold %s", (long long)pc, (long long)r, want);
    return err;
  }
  bool get_int(int64_t r, int64_t* v) {
    const Ref& o = reg(r);
    if (o && o->kind == Object::kInt) {
      *v = o->ival;
      return true;
    }
    if (o && o->kind == Object::kTensor && o->on_host && elements(*o) == 1) {
      *v = static_cast<const int64_t*>(o->data)[0];
      return true;
    }
    bad(r, "an integer");
    return false;
  }
  Object* get_tensor(int64_t r, bool host) {
    const Ref& o = reg(r);
    if (!o || o->kind != Object::kTensor || o->on_host != host) {
      bad(r, host ? "a host shape tensor" : "a GPU tensor");
      return nullptr;
    }
    if (o->storage && o->storage->freed) {
      err = fail(NIMBLE_ERR_ARG, "pc %lld: register %lld refers to storage that was freed", (long long)pc, (long long)r);
      return nullptr;
    }
    return o.get();
  }
  Object* get_shape(int64_t r) {
    Object* o = get_tensor(r, true);
    if (o && (o->rank != 1 || o->shape[0] > kMaxRank)) {
      bad(r, "a rank-1 shape tensor of at most 4 extents");
      return nullptr;
    }
    return o;
  }
};

bool same_shape(const Object& t, const int64_t* shape, int rank) {
  if (t.rank != rank) return false;
  for (int i = 0; i < rank; ++i)
    if (t.shape[i] != shape[i]) return false;
  return true;
}

int invoke_packed(Frame& f, int id, const int64_t* r) {
  nimble_vm* vm = f.vm;
  switch (id) {
    case NIMBLE_PF_SHAPE_DENSE: {
      Object *x = f.get_shape(r[0]), *w = f.get_shape(r[1]), *o = f.get_shape(r[2]);
      if (!x || !w || !o) return f.err;
      if (o->shape[0] != 2) return f.bad(r[2], "a shape tensor of 2 extents");
      return nimble_dense_shape(static_cast<int64_t*>(x->data), (int)x->shape[0],
                                static_cast<int64_t*>(w->data), (int)w->shape[0],
                                static_cast<int64_t*>(o->data));
    }
    case NIMBLE_PF_SHAPE_LSTM: {
      Object* in[4];
      for (int i = 0; i < 4; ++i) {
        in[i] = f.get_shape(r[i]);
        if (!in[i]) return f.err;
        if (in[i]->shape[0] != 2) return f.bad(r[i], "the shape of a rank-2 tensor");
      }
      Object *ho = f.get_shape(r[4]), *co = f.get_shape(r[5]);
      if (!ho || !co) return f.err;
      if (ho->shape[0] != 2) return f.bad(r[4], "a shape tensor of 2 extents");
      if (co->shape[0] != 2) return f.bad(r[5], "a shape tensor of 2 extents");
      return nimble_lstm_shape(static_cast<int64_t*>(in[0]->data), static_cast<int64_t*>(in[1]->data),
                               static_cast<int64_t*>(in[2]->data), static_cast<int64_t*>(in[3]->data),
                               static_cast<int64_t*>(ho->data), static_cast<int64_t*>(co->data));
    }
    case NIMBLE_PF_SHAPE_ATTENTION: {
      Object *q = f.get_shape(r[0]), *k = f.get_shape(r[1]), *v = f.get_shape(r[2]), *o = f.get_shape(r[3]);
      if (!q || !k || !v || !o) return f.err;
      if (o->shape[0] != 3) return f.bad(r[3], "a shape tensor of 3 extents");
      int64_t s[3];
      int rc = nimble_batch_matmul_shape(static_cast<int64_t*>(q->data), (int)q->shape[0],
                                         static_cast<int64_t*>(k->data), (int)k->shape[0], 1, s);
      if (rc != NIMBLE_OK) return rc;
      return nimble_batch_matmul_shape(s, 3, static_cast<int64_t*>(v->data), (int)v->shape[0], 0,
                                       static_cast<int64_t*>(o->data));
    }
    case NIMBLE_PF_STORAGE_BYTES: {
      Object* s = f.get_shape(r[0]);
      int64_t dtype;
      if (!s || !f.get_int(r[1], &dtype)) return f.err;
      if (dtype_size((int)dtype) == 0) return fail(NIMBLE_ERR_DTYPE, "pc %lld: unknown dtype %lld", (long long)f.pc, (long long)dtype);
      int64_t n = dtype == NIMBLE_I64 ? 8 : 0;
      if (dtype == NIMBLE_I64) {
        for (int i = 0; i < s->shape[0]; ++i) n *= static_cast<int64_t*>(s->data)[i];
      } else {
        n = nimble_storage_bytes(static_cast<int64_t*>(s->data), (int)s->shape[0], (int)dtype);
        if (n < 0) return (int)n;
      }
      vm->regs[r[2]] = make_int(n);
      return NIMBLE_OK;
    }
    case NIMBLE_PF_SHAPE_GET: {
      Object* s = f.get_shape(r[0]);
      int64_t i;
      if (!s || !f.get_int(r[1], &i)) return f.err;
      if (i < 0 || i >= s->shape[0]) return fail(NIMBLE_ERR_ARG, "pc %lld: extent %lld of a rank-%lld shape", (long long)f.pc, (long long)i, (long long)s->shape[0]);
      vm->regs[r[2]] = make_int(static_cast<int64_t*>(s->data)[i]);
      return NIMBLE_OK;
    }
    case NIMBLE_PF_INT_ADD:
    case NIMBLE_PF_INT_LESS: {
      int64_t a, b;
      if (!f.get_int(r[0], &a) || !f.get_int(r[1], &b)) return f.err;
      vm->regs[r[2]] = make_int(id == NIMBLE_PF_INT_ADD ? a + b : (a < b ? 1 : 0));
      return NIMBLE_OK;
    }
    case NIMBLE_PF_INDEX0: {
      Object* t = f.get_tensor(r[0], false);
      int64_t i;
      if (!t || !f.get_int(r[1], &i)) return f.err;
      if (t->rank < 1 || i < 0 || i >= t->shape[0])
        return fail(NIMBLE_ERR_ARG, "pc %lld: slice %lld of a tensor with leading extent %lld", (long long)f.pc, (long long)i, (long long)(t->rank ? t->shape[0] : 0));
      auto v = std::make_shared<Object>(*t);
      v->rank = t->rank - 1;
      int64_t inner = 1;
      for (int d = 1; d < t->rank; ++d) {
        v->shape[d - 1] = t->shape[d];
        inner *= t->shape[d];
      }
      v->shape[v->rank] = 0;
      v->data = static_cast<char*>(t->data) + i * inner * dtype_size(t->dtype);
      vm->regs[r[2]] = v;
      return NIMBLE_OK;
    }
    case NIMBLE_PF_DENSE:
    case NIMBLE_PF_DENSE_BIAS:
    case NIMBLE_PF_DENSE_BIAS_GELU: {
      const bool has_bias = id != NIMBLE_PF_DENSE;
      Object *x = f.get_tensor(r[0], false), *w = f.get_tensor(r[1], false);
      Object* b = has_bias ? f.get_tensor(r[2], false) : nullptr;
      Object* y = f.get_tensor(r[has_bias ? 3 : 2], false);
      if (!x || !w || (has_bias && !b) || !y) return f.err;
      int64_t out[2];
      int rc = nimble_dense_shape(x->shape, x->rank, w->shape, w->rank, out);
      if (rc != NIMBLE_OK) return rc;
      if (x->dtype != NIMBLE_BF16 || w->dtype != NIMBLE_BF16 || (b && b->dtype != NIMBLE_BF16))
        return fail(NIMBLE_ERR_DTYPE, "pc %lld: dense operands must be bf16", (long long)f.pc);
      if (b && (b->rank != 1 || b->shape[0] != out[1]))
        return fail(NIMBLE_ERR_SHAPE, "pc %lld: bias is not [N]", (long long)f.pc);
      if (!same_shape(*y, out, 2))
        return fail(NIMBLE_ERR_SHAPE, "pc %lld: output tensor is not the [M,N] the shape function gives", (long long)f.pc);
      const int epi = id == NIMBLE_PF_DENSE ? NIMBLE_EPI_NONE
                      : id == NIMBLE_PF_DENSE_BIAS ? NIMBLE_EPI_BIAS : NIMBLE_EPI_BIAS_GELU_ERF;
      return nimble_dense_dyn(x->data, w->data, b ? b->data : nullptr, y->data, out[0], out[1],
                              x->shape[1], epi, y->dtype, vm->workspace, vm->workspace_bytes, vm->stream);
    }
    case NIMBLE_PF_LSTM_GATES: {
      Object* t[7];
      for (int i = 0; i < 7; ++i) {
        t[i] = f.get_tensor(r[i], false);
        if (!t[i]) return f.err;
      }
      Object *x = t[0], *h = t[1], *w = t[2], *b = t[3], *c = t[4], *co = t[5], *ho = t[6];
      if (x->rank != 2 || h->rank != 2 || c->rank != 2 || w->rank != 2)
        return fail(NIMBLE_ERR_RANK, "pc %lld: lstm_gates operands must have rank 2", (long long)f.pc);
      int64_t hs[2], cs[2];
      int rc = nimble_lstm_shape(x->shape, h->shape, c->shape, w->shape, hs, cs);
      if (rc != NIMBLE_OK) return rc;
      if (x->dtype != NIMBLE_BF16 || h->dtype != NIMBLE_BF16 || w->dtype != NIMBLE_BF16 ||
          b->dtype != NIMBLE_BF16 || c->dtype != NIMBLE_F32 || co->dtype != NIMBLE_F32 || ho->dtype != NIMBLE_BF16)
        return fail(NIMBLE_ERR_DTYPE, "pc %lld: lstm_gates takes bf16 x, h, w, b and h', f32 c and c'", (long long)f.pc);
      if (b->rank != 1 || b->shape[0] != w->shape[0])
        return fail(NIMBLE_ERR_SHAPE, "pc %lld: bias is not [4H]", (long long)f.pc);
      if (!same_shape(*ho, hs, 2) || !same_shape(*co, cs, 2))
        return fail(NIMBLE_ERR_SHAPE, "pc %lld: output tensors are not the [B,H] the shape function gives", (long long)f.pc);
      return nimble_lstm_gates_dyn(x->data, h->data, w->data, b->data, c->data, co->data, ho->data,
                                   x->shape[0], x->shape[1], h->shape[1], vm->workspace,
                                   vm->workspace_bytes, vm->stream);
    }
    case NIMBLE_PF_ATTENTION: {
      Object* t[4];
      for (int i = 0; i < 4; ++i) {
        t[i] = f.get_tensor(r[i], false);
        if (!t[i]) return f.err;
        if (t[i]->dtype != NIMBLE_BF16) return fail(NIMBLE_ERR_DTYPE, "pc %lld: attention operands must be bf16", (long long)f.pc);
      }
      int64_t s[3], o[3];
      int rc = nimble_batch_matmul_shape(t[0]->shape, t[0]->rank, t[1]->shape, t[1]->rank, 1, s);
      if (rc == NIMBLE_OK) rc = nimble_batch_matmul_shape(s, 3, t[2]->shape, t[2]->rank, 0, o);
      if (rc != NIMBLE_OK) return rc;
      if (s[1] != s[2]) return fail(NIMBLE_ERR_SHAPE, "pc %lld: q and k lengths differ", (long long)f.pc);
      if (!same_shape(*t[3], o, 3))
        return fail(NIMBLE_ERR_SHAPE, "pc %lld: output tensor is not the [T,L,D] the shape function gives", (long long)f.pc);
      const int64_t D = t[0]->shape[2];
      return nimble_attention_dyn(t[0]->data, t[1]->data, t[2]->data, t[3]->data, o[0], o[1], D,
                                  1.0f / std::sqrt((float)D), vm->stream);
    }
    default:
      return fail(NIMBLE_ERR_ARG, "pc %lld: unknown packed function %d", (long long)f.pc, id);
  }
}

bool flatten(const Ref& o, std::vector<nimble_vm_tensor>* out) {
  if (!o) return false;
  nimble_vm_tensor t;
  std::memset(&t, 0, sizeof(t));
  switch (o->kind) {
    case Object::kInt:
      t.dtype = NIMBLE_I64;
      t.rank = 0;
      t.shape[0] = o->ival;
      out->push_back(t);
      return true;
    case Object::kTensor:
      t.data = o->data;
      t.dtype = o->dtype;
      t.rank = o->rank;
      for (int i = 0; i < o->rank; ++i) t.shape[i] = o->shape[i];
      out->push_back(t);
      return true;
    case Object::kAdt:
      for (const Ref& fld : o->fields)
        if (!flatten(fld, out)) return false;
      return true;
    default:
      return false;
  }
}

}  // namespace

extern "C" {

int nimble_vm_create(const int64_t* code, int64_t n_words, int64_t n_registers,
                     const nimble_vm_tensor* constants, int n_constants, nimble_vm** out) {
  nimble::clear_error();
  if (!code || !out || (n_constants > 0 && !constants)) return fail(NIMBLE_ERR_NULL, "vm_create: null argument");
  if (n_words <= 0 || n_registers <= 0 || n_registers > (1 << 20) || n_constants < 0)
    return fail(NIMBLE_ERR_ARG, "vm_create: empty code or bad register/constant count");
  std::unique_ptr<nimble_vm> vm(new nimble_vm);
  vm->n_registers = n_registers;
  for (int i = 0; i < n_constants; ++i) {
    int err = 0;
    Ref c = from_boundary(constants[i], &err, "constant", i);
    if (!c) return err;
    vm->constants.push_back(c);
  }
  // decode
  int64_t at = 0;
  while (at < n_words) {
    if (at + 2 > n_words) return fail(NIMBLE_ERR_ARG, "vm_create: truncated instruction at word %lld", (long long)at);
    const int64_t op = code[at], n = code[at + 1];
    if (op < 0 || op >= NIMBLE_OP_COUNT) return fail(NIMBLE_ERR_ARG, "vm_create: unknown opcode %lld at word %lld", (long long)op, (long long)at);
    if (n < 0 || at + 2 + n > n_words) return fail(NIMBLE_ERR_ARG, "vm_create: %s at word %lld runs past the end", kOpNames[op], (long long)at);
    Instr in;
    in.op = (int)op;
    in.a.assign(code + at + 2, code + at + 2 + n);
    vm->code.push_back(std::move(in));
    at += 2 + n;
  }
  // verify
  const int64_t count = (int64_t)vm->code.size();
  auto is_reg = [&](int64_t r) { return r >= 0 && r < n_registers; };
  for (int64_t pc = 0; pc < count; ++pc) {
    const Instr& in = vm->code[pc];
    const std::vector<int64_t>& a = in.a;
    const int64_t n = (int64_t)a.size();
    const char* name = kOpNames[in.op];
    if (kOperands[in.op] == -2) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: %s is not implemented by this interpreter", (long long)pc, name);
    if (kOperands[in.op] >= 0 && n != kOperands[in.op])
      return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: %s takes %d operands, got %lld", (long long)pc, name, kOperands[in.op], (long long)n);
    bool regs_ok = true, falls = true;
    auto jump_ok = [&](int64_t off) { return pc + off >= 0 && pc + off < count; };
    switch (in.op) {
      case NIMBLE_OP_MOVE: regs_ok = is_reg(a[0]) && is_reg(a[1]); break;
      case NIMBLE_OP_RET: regs_ok = is_reg(a[0]); falls = false; break;
      case NIMBLE_OP_IF:
        regs_ok = is_reg(a[0]) && is_reg(a[1]);
        if (!jump_ok(a[2]) || !jump_ok(a[3])) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: If jumps outside the function", (long long)pc);
        falls = false;
        break;
      case NIMBLE_OP_GOTO:
        if (!jump_ok(a[0])) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: Goto jumps outside the function", (long long)pc);
        falls = false;
        break;
      case NIMBLE_OP_LOAD_CONST:
        if (a[0] < 0 || a[0] >= n_constants) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: constant %lld of %d", (long long)pc, (long long)a[0], n_constants);
        regs_ok = is_reg(a[1]);
        break;
      case NIMBLE_OP_LOAD_CONSTI: regs_ok = is_reg(a[1]); break;
      case NIMBLE_OP_ALLOC_STORAGE:
        regs_ok = is_reg(a[0]) && is_reg(a[3]);
        if (a[1] <= 0 || (a[1] & (a[1] - 1)) || a[1] > 4096) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: alignment %lld is not a power of two up to 4096", (long long)pc, (long long)a[1]);
        if (a[2] != 0 && a[2] != 1) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: device %lld (0 host, 1 GPU)", (long long)pc, (long long)a[2]);
        break;
      case NIMBLE_OP_ALLOC_TENSOR:
        if (n < 5 || a[3] < 0 || a[3] > kMaxRank || n != 5 + a[3]) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: malformed AllocTensor", (long long)pc);
        if (dtype_size((int)a[2]) == 0 || a[1] < 0) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: AllocTensor dtype or offset", (long long)pc);
        for (int64_t i = 0; i < a[3]; ++i)
          if (a[4 + i] < 0) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: negative extent", (long long)pc);
        regs_ok = is_reg(a[0]) && is_reg(a[n - 1]);
        break;
      case NIMBLE_OP_ALLOC_TENSOR_REG:
        if (dtype_size((int)a[3]) == 0 || a[1] < 0) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: AllocTensorReg dtype or offset", (long long)pc);
        regs_ok = is_reg(a[0]) && is_reg(a[2]) && is_reg(a[4]);
        break;
      case NIMBLE_OP_ALLOC_ADT:
        if (n < 3 || a[1] < 0 || n != 3 + a[1]) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: malformed AllocADT", (long long)pc);
        for (int64_t i = 0; i <= a[1]; ++i) regs_ok = regs_ok && is_reg(a[2 + i]);
        break;
      case NIMBLE_OP_FREE_STORAGE:
      case NIMBLE_OP_FREE_TENSOR: regs_ok = is_reg(a[0]); break;
      case NIMBLE_OP_INVOKE_PACKED: {
        if (n < 3 || a[0] < 0 || a[0] >= NIMBLE_PF_COUNT) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: unknown packed function", (long long)pc);
        const PackedInfo& pf = kPacked[a[0]];
        if (a[1] != pf.inputs + pf.outputs || a[2] != pf.outputs || n != 3 + a[1])
          return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: %s takes %d inputs and %d outputs", (long long)pc, pf.name, pf.inputs, pf.outputs);
        for (int64_t i = 0; i < a[1]; ++i) regs_ok = regs_ok && is_reg(a[3 + i]);
        break;
      }
      case NIMBLE_OP_GET_FIELD:
        regs_ok = is_reg(a[0]) && is_reg(a[2]);
        if (a[1] < 0) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: negative field index", (long long)pc);
        break;
      case NIMBLE_OP_GET_TAG:
      case NIMBLE_OP_SHAPE_OF: regs_ok = is_reg(a[0]) && is_reg(a[1]); break;
      case NIMBLE_OP_RESHAPE_TENSOR: regs_ok = is_reg(a[0]) && is_reg(a[1]) && is_reg(a[2]); break;
      case NIMBLE_OP_FATAL: falls = false; break;
      default: break;
    }
    if (!regs_ok) return fail(NIMBLE_ERR_ARG, "vm_create: instruction %lld: %s names a register outside 0..%lld", (long long)pc, name, (long long)n_registers - 1);
    if (falls && pc + 1 >= count) return fail(NIMBLE_ERR_ARG, "vm_create: the function runs off its end after instruction %lld (%s)", (long long)pc, name);
  }
  vm->regs.resize(n_registers);
  *out = vm.release();
  return NIMBLE_OK;
}

void nimble_vm_destroy(nimble_vm* vm) { delete vm; }

int nimble_vm_run(nimble_vm* vm, const nimble_vm_tensor* inputs, int n_inputs, void* pool,
                  uint64_t pool_bytes, void* workspace, uint64_t workspace_bytes, void* stream,
                  int64_t max_instructions, nimble_vm_tensor* results, int max_results,
                  int* n_results) {
  nimble::clear_error();
  if (!vm || !n_results || (n_inputs > 0 && !inputs) || (max_results > 0 && !results))
    return fail(NIMBLE_ERR_NULL, "vm_run: null argument");
  if (n_inputs < 0 || n_inputs > vm->n_registers) return fail(NIMBLE_ERR_ARG, "vm_run: %d inputs for %lld registers", n_inputs, (long long)vm->n_registers);
  if (pool_bytes > 0 && !pool) return fail(NIMBLE_ERR_NULL, "vm_run: null pool");
  if (reinterpret_cast<uintptr_t>(pool) % 64) return fail(NIMBLE_ERR_ALIGN, "vm_run: the pool must be 64-byte aligned");
  *n_results = 0;
  vm->result.reset();
  for (Ref& r : vm->regs) r.reset();
  vm->pool.reset(pool, pool_bytes);
  vm->workspace = workspace;
  vm->workspace_bytes = workspace_bytes;
  vm->stream = stream;
  std::memset(vm->op_count, 0, sizeof(vm->op_count));
  std::memset(vm->op_ns, 0, sizeof(vm->op_ns));
  std::memset(vm->pf_count, 0, sizeof(vm->pf_count));
  std::memset(vm->pf_ns, 0, sizeof(vm->pf_ns));
  for (int i = 0; i < n_inputs; ++i) {
    int err = 0;
    vm->regs[i] = from_boundary(inputs[i], &err, "input", i);
    if (!vm->regs[i]) return err;
  }
  const int64_t limit = max_instructions > 0 ? max_instructions : kDefaultInstructionLimit;
  const int64_t count = (int64_t)vm->code.size();
  Frame f{vm, 0};
  int64_t executed = 0;
  int rc = NIMBLE_OK;
  bool done = false;
  using clock = std::chrono::steady_clock;
  while (!done) {
    if (executed++ >= limit) {
      rc = fail(NIMBLE_ERR_ARG, "vm_run: instruction limit of %lld reached at pc %lld", (long long)limit, (long long)f.pc);
      break;
    }
    const Instr& in = vm->code[f.pc];
    const int64_t* a = in.a.data();
    const auto t0 = clock::now();
    int64_t next = f.pc + 1;
    int pf = -1;
    switch (in.op) {
      case NIMBLE_OP_MOVE: vm->regs[a[1]] = vm->regs[a[0]]; break;
      case NIMBLE_OP_RET:
        vm->result = vm->regs[a[0]];
        done = true;
        break;
      case NIMBLE_OP_IF: {
        int64_t t, u;
        if (!f.get_int(a[0], &t) || !f.get_int(a[1], &u)) { rc = f.err; break; }
        next = f.pc + (t == u ? a[2] : a[3]);
        break;
      }
      case NIMBLE_OP_GOTO: next = f.pc + a[0]; break;
      case NIMBLE_OP_LOAD_CONST: vm->regs[a[1]] = vm->constants[a[0]]; break;
      case NIMBLE_OP_LOAD_CONSTI: vm->regs[a[1]] = make_int(a[0]); break;
      case NIMBLE_OP_ALLOC_STORAGE: {
        int64_t size;
        if (!f.get_int(a[0], &size)) { rc = f.err; break; }
        if (size < 0) { rc = fail(NIMBLE_ERR_ARG, "pc %lld: negative storage size", (long long)f.pc); break; }
        auto st = std::make_shared<Storage>();
        if (a[2] == 0) {
          st->host.assign((size_t)((size + 7) / 8), 0);
          st->bytes = (uint64_t)size;
        } else {
          // block sizes are multiples of the larger of the requested alignment and 64 bytes
          const uint64_t align = a[1] > 64 ? (uint64_t)a[1] : 64u;
          uint64_t want = ((uint64_t)size + align - 1) / align * align;
          if (want == 0) want = align;
          uint64_t off, got;
          if (!vm->pool.take(want, align, &off, &got)) {
            rc = fail(NIMBLE_ERR_WORKSPACE, "pc %lld: device pool exhausted: %llu bytes wanted, %llu of %llu in use", (long long)f.pc,
                      (unsigned long long)want, (unsigned long long)vm->pool.top, (unsigned long long)vm->pool.bytes);
            break;
          }
          st->device = true;
          st->offset = off;
          st->bytes = got;
          st->pool = &vm->pool;
          st->generation = vm->pool.generation;
        }
        auto o = std::make_shared<Object>();
        o->kind = Object::kStorage;
        o->storage = st;
        vm->regs[a[3]] = o;
        break;
      }
      case NIMBLE_OP_ALLOC_TENSOR:
      case NIMBLE_OP_ALLOC_TENSOR_REG: {
        const Ref& so = vm->regs[a[0]];
        if (!so || so->kind != Object::kStorage) { rc = f.bad(a[0], "a storage"); break; }
        if (so->storage->freed) { rc = fail(NIMBLE_ERR_ARG, "pc %lld: storage in register %lld was freed", (long long)f.pc, (long long)a[0]); break; }
        auto t = std::make_shared<Object>();
        t->kind = Object::kTensor;
        int64_t dst;
        if (in.op == NIMBLE_OP_ALLOC_TENSOR) {
          t->dtype = (int)a[2];
          t->rank = (int)a[3];
          for (int i = 0; i < t->rank; ++i) t->shape[i] = a[4 + i];
          dst = a[4 + t->rank];
        } else {
          Object* sh = f.get_shape(a[2]);
          if (!sh) { rc = f.err; break; }
          t->dtype = (int)a[3];
          t->rank = (int)sh->shape[0];
          bool neg = false;
          for (int i = 0; i < t->rank; ++i) {
            t->shape[i] = static_cast<int64_t*>(sh->data)[i];
            neg = neg || t->shape[i] < 0;
          }
          if (neg) { rc = fail(NIMBLE_ERR_ARG, "pc %lld: negative extent in the shape register", (long long)f.pc); break; }
          dst = a[4];
        }
        const Storage& st = *so->storage;
        const uint64_t need = (uint64_t)(elements(*t) * dtype_size(t->dtype));
        if ((uint64_t)a[1] + need > st.bytes) {
          rc = fail(NIMBLE_ERR_WORKSPACE, "pc %lld: tensor of %llu bytes at offset %lld does not fit its storage of %llu bytes", (long long)f.pc,
                    (unsigned long long)need, (long long)a[1], (unsigned long long)st.bytes);
          break;
        }
        if (st.device) {
          if (t->dtype == NIMBLE_I64) { rc = fail(NIMBLE_ERR_DTYPE, "pc %lld: shape tensors live in host storage", (long long)f.pc); break; }
          if (a[1] % 16) { rc = fail(NIMBLE_ERR_ALIGN, "pc %lld: tensor offset %lld is not 16-byte aligned", (long long)f.pc, (long long)a[1]); break; }
          t->data = vm->pool.base + st.offset + a[1];
        } else {
          if (t->dtype != NIMBLE_I64 || a[1] % 8) { rc = fail(NIMBLE_ERR_DTYPE, "pc %lld: host storage holds i64 shape tensors only", (long long)f.pc); break; }
          t->data = so->storage->host.data() + a[1] / 8;
          t->on_host = true;
        }
        t->storage = so->storage;
        vm->regs[dst] = t;
        break;
      }
      case NIMBLE_OP_ALLOC_ADT: {
        auto o = std::make_shared<Object>();
        o->kind = Object::kAdt;
        o->ival = a[0];
        for (int64_t i = 0; i < a[1]; ++i) {
          if (!vm->regs[a[2 + i]]) { rc = f.bad(a[2 + i], "an object"); break; }
          o->fields.push_back(vm->regs[a[2 + i]]);
        }
        if (rc == NIMBLE_OK) vm->regs[a[2 + a[1]]] = o;
        break;
      }
      case NIMBLE_OP_FREE_STORAGE: {
        const Ref& so = vm->regs[a[0]];
        if (!so || so->kind != Object::kStorage) { rc = f.bad(a[0], "a storage"); break; }
        so->storage->release();
        break;
      }
      case NIMBLE_OP_FREE_TENSOR: {
        const Ref& t = vm->regs[a[0]];
        if (!t || t->kind != Object::kTensor) { rc = f.bad(a[0], "a tensor"); break; }
        vm->regs[a[0]].reset();
        break;
      }
      case NIMBLE_OP_INVOKE_PACKED:
        pf = (int)a[0];
        rc = invoke_packed(f, pf, a + 3);
        break;
      case NIMBLE_OP_GET_FIELD: {
        const Ref& o = vm->regs[a[0]];
        if (!o || o->kind != Object::kAdt) { rc = f.bad(a[0], "an ADT"); break; }
        if (a[1] >= (int64_t)o->fields.size()) { rc = fail(NIMBLE_ERR_ARG, "pc %lld: field %lld of an ADT with %zu fields", (long long)f.pc, (long long)a[1], o->fields.size()); break; }
        vm->regs[a[2]] = o->fields[a[1]];
        break;
      }
      case NIMBLE_OP_GET_TAG: {
        const Ref& o = vm->regs[a[0]];
        if (!o || o->kind != Object::kAdt) { rc = f.bad(a[0], "an ADT"); break; }
        vm->regs[a[1]] = make_int(o->ival);
        break;
      }
      case NIMBLE_OP_SHAPE_OF: {
        const Ref& t = vm->regs[a[0]];
        if (!t || t->kind != Object::kTensor) { rc = f.bad(a[0], "a tensor"); break; }
        vm->regs[a[1]] = make_host_shape(t->shape, t->rank);
        break;
      }
      case NIMBLE_OP_RESHAPE_TENSOR: {
        const Ref& t = vm->regs[a[0]];
        if (!t || t->kind != Object::kTensor) { rc = f.bad(a[0], "a tensor"); break; }
        Object* sh = f.get_shape(a[1]);
        if (!sh) { rc = f.err; break; }
        auto v = std::make_shared<Object>(*t);
        v->rank = (int)sh->shape[0];
        for (int i = 0; i < kMaxRank; ++i) v->shape[i] = i < v->rank ? static_cast<int64_t*>(sh->data)[i] : 0;
        bool neg = false;
        for (int i = 0; i < v->rank; ++i) neg = neg || v->shape[i] < 0;
        if (neg || elements(*v) != elements(*t)) { rc = fail(NIMBLE_ERR_SHAPE, "pc %lld: reshape changes the element count", (long long)f.pc); break; }
        vm->regs[a[2]] = v;
        break;
      }
      case NIMBLE_OP_FATAL:
        rc = fail(NIMBLE_ERR_SHAPE, "pc %lld: Fatal", (long long)f.pc);
        break;
      default:
        rc = fail(NIMBLE_ERR_ARG, "pc %lld: opcode %d not implemented", (long long)f.pc, in.op);
        break;
    }
    const int64_t ns = std::chrono::duration_cast<std::chrono::nanoseconds>(clock::now() - t0).count();
    vm->op_count[in.op] += 1;
    vm->op_ns[in.op] += ns;
    if (pf >= 0) {
      vm->pf_count[pf] += 1;
      vm->pf_ns[pf] += ns;
    }
    if (rc != NIMBLE_OK) break;
    f.pc = next;
    if (!done && (f.pc < 0 || f.pc >= count)) {  // unreachable after the load-time check
      rc = fail(NIMBLE_ERR_ARG, "vm_run: pc %lld outside the function", (long long)f.pc);
      break;
    }
  }
  // registers are dropped; only the result keeps its storage alive
  for (Ref& r : vm->regs) r.reset();
  if (rc != NIMBLE_OK) {
    vm->result.reset();
    return rc;
  }
  std::vector<nimble_vm_tensor> flat;
  if (!flatten(vm->result, &flat)) return fail(NIMBLE_ERR_ARG, "vm_run: the result register holds no tensor, integer or ADT of those");
  if ((int)flat.size() > max_results) return fail(NIMBLE_ERR_ARG, "vm_run: %zu results, room for %d", flat.size(), max_results);
  for (size_t i = 0; i < flat.size(); ++i) results[i] = flat[i];
  *n_results = (int)flat.size();
  return NIMBLE_OK;
}

int nimble_vm_profile(const nimble_vm* vm, int64_t* op_count, int64_t* op_ns,
                      int64_t* packed_count, int64_t* packed_ns, uint64_t* pool_high_water,
                      int64_t* storage_allocs, int64_t* storage_reuses) {
  if (!vm) return fail(NIMBLE_ERR_NULL, "vm_profile: null vm");
  if (op_count) std::memcpy(op_count, vm->op_count, sizeof(vm->op_count));
  if (op_ns) std::memcpy(op_ns, vm->op_ns, sizeof(vm->op_ns));
  if (packed_count) std::memcpy(packed_count, vm->pf_count, sizeof(vm->pf_count));
  if (packed_ns) std::memcpy(packed_ns, vm->pf_ns, sizeof(vm->pf_ns));
  if (pool_high_water) *pool_high_water = vm->pool.high_water;
  if (storage_allocs) *storage_allocs = vm->pool.allocs;
  if (storage_reuses) *storage_reuses = vm->pool.reuses;
  return NIMBLE_OK;
}

}  // extern "C"
