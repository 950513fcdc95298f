/* Recording fast path of the Python binding (CPython extension `_ltrec`).
 *
 * Recording an op is the hot path of the method on the host (section 3: every tensor operation of
 * the user's program becomes one call), and a ctypes call costs several times what lt_op itself
 * does.  This module makes the same C-ABI calls -- lt_scalar for Python numbers among the
 * operands, lt_op, lt_release for those temporaries, lt_assign -- from C, and defines the
 * binding's tensor handle as a C type, so that recording an op creates and destroys no Python
 * frames beyond the caller's.  It holds no state of the method and links against nothing: the
 * binding passes the addresses of the entry points once.
 */
#define PY_SSIZE_T_CLEAN
#include <Python.h>
#include <stdint.h>
#include <structmember.h>

typedef int (*lt_op_fn)(void* ctx, uint16_t opcode, const uint64_t* inputs, int n_in, const void* attrs, int n_attr,
                        uint64_t* outputs, int n_out);
typedef int (*lt_scalar_fn)(void* ctx, int dtype, double value, uint64_t* out);
typedef int (*lt_release_fn)(void* ctx, uint64_t t);
typedef const char* (*lt_last_error_fn)(void* ctx);
typedef int (*lt_assign_fn)(void* ctx, uint64_t dst, uint64_t src);
typedef int (*lt_release_many_fn)(void* ctx, const uint64_t* ids, size_t n);
typedef int (*lt_barrier_fn)(void* ctx, int blocking, void* info);

static lt_op_fn p_op;
static lt_scalar_fn p_scalar;
static lt_release_fn p_release;
static lt_last_error_fn p_last_error;
static lt_assign_fn p_assign;
static lt_release_many_fn p_release_many;
static lt_barrier_fn p_barrier;
static PyObject* str_tid;
static PyObject* str_dead;
static PyObject* str_kept;
static PyObject* rec_error;
static PyObject* query_hook;   /* callable(tensor): fills in _dtype and _shape from the library */

enum { kMaxIn = 8, kMaxOut = 4 };

/* ---- the tensor handle -------------------------------------------------------------------
 * A unique tensor id plus what the binding knows about it.  Dropping the last reference tells the
 * context that the tensor is no longer live: the id is appended to the context's `_dead` list,
 * which the binding hands to lt_release_many before anything that looks at liveness.  Element type
 * and shape of an op's result are asked from the library only when somebody reads them. */
typedef struct {
  PyObject_HEAD
  PyObject* ctx;     /* the binding's Context; None once released by hand */
  unsigned long long tid;
  PyObject* dtype;   /* str, or None: not asked yet */
  PyObject* shape;   /* tuple, or None */
  PyObject* keep;    /* owner of the device buffer behind a leaf, or None */
  PyObject* weakrefs;
} TensorObject;

static PyTypeObject TensorType;

static PyObject* tensor_make(PyObject* ctx, unsigned long long tid) {
  TensorObject* t = PyObject_New(TensorObject, &TensorType);
  if (!t) return NULL;
  Py_INCREF(ctx);
  t->ctx = ctx;
  t->tid = tid;
  Py_INCREF(Py_None); t->dtype = Py_None;
  Py_INCREF(Py_None); t->shape = Py_None;
  Py_INCREF(Py_None); t->keep = Py_None;
  t->weakrefs = NULL;
  return (PyObject*)t;
}

static PyObject* tensor_new(PyTypeObject* type, PyObject* args, PyObject* kw) {
  static char* names[] = {"ctx", "tid", "dtype", "shape", "keep", NULL};
  PyObject *ctx, *dtype = Py_None, *shape = Py_None, *keep = Py_None;
  unsigned long long tid;
  if (!PyArg_ParseTupleAndKeywords(args, kw, "OK|OOO", names, &ctx, &tid, &dtype, &shape, &keep)) return NULL;
  PyObject* shp;
  if (shape == Py_None) {
    Py_INCREF(Py_None);
    shp = Py_None;
  } else {
    shp = PySequence_Tuple(shape);
    if (!shp) return NULL;
  }
  TensorObject* t = (TensorObject*)tensor_make(ctx, tid);
  if (!t) {
    Py_DECREF(shp);
    return NULL;
  }
  Py_INCREF(dtype); Py_SETREF(t->dtype, dtype);
  Py_SETREF(t->shape, shp);
  Py_INCREF(keep); Py_SETREF(t->keep, keep);
  return (PyObject*)t;
}

static void tensor_dealloc(TensorObject* self) {
  if (self->weakrefs) PyObject_ClearWeakRefs((PyObject*)self);
  if (self->ctx && self->ctx != Py_None) {
    PyObject *et, *ev, *tb;
    PyErr_Fetch(&et, &ev, &tb);
    PyObject* dead = PyObject_GetAttr(self->ctx, str_dead);
    if (dead && PyList_Check(dead)) {
      PyObject* id = PyLong_FromUnsignedLongLong(self->tid);
      if (id) {
        (void)PyList_Append(dead, id);
        Py_DECREF(id);
      }
    }
    Py_XDECREF(dead);
    /* the trace being recorded may still name this leaf's device memory (its device_data node holds
     * the raw pointer until the next barrier has run): the owner of that memory moves to the
     * context's `_kept` list, which the binding empties once the barrier has been enqueued */
    if (self->keep && self->keep != Py_None) {
      PyObject* kept = PyObject_GetAttr(self->ctx, str_kept);
      if (kept && PyList_Check(kept)) (void)PyList_Append(kept, self->keep);
      Py_XDECREF(kept);
    }
    PyErr_Clear();   /* a destructor has nobody to report to */
    PyErr_Restore(et, ev, tb);
  }
  Py_XDECREF(self->ctx);
  Py_XDECREF(self->dtype);
  Py_XDECREF(self->shape);
  Py_XDECREF(self->keep);
  Py_TYPE(self)->tp_free((PyObject*)self);
}

static int tensor_ask(TensorObject* self) {   /* 0: _dtype and _shape are known now */
  if (!query_hook) {
    PyErr_SetString(PyExc_RuntimeError, "_ltrec.set_query has not been called");
    return -1;
  }
  PyObject* r = PyObject_CallFunctionObjArgs(query_hook, (PyObject*)self, NULL);
  if (!r) return -1;
  Py_DECREF(r);
  return 0;
}

static PyObject* tensor_get_dtype(TensorObject* self, void* closure) {
  if (self->dtype == Py_None && tensor_ask(self) < 0) return NULL;
  Py_INCREF(self->dtype);
  return self->dtype;
}

static int tensor_set_dtype(TensorObject* self, PyObject* v, void* closure) {
  if (!v) v = Py_None;
  Py_INCREF(v);
  Py_SETREF(self->dtype, v);
  return 0;
}

static PyObject* tensor_get_shape(TensorObject* self, void* closure) {
  if (self->shape == Py_None && tensor_ask(self) < 0) return NULL;
  Py_INCREF(self->shape);
  return self->shape;
}

static int tensor_set_shape(TensorObject* self, PyObject* v, void* closure) {
  PyObject* shp;
  if (!v || v == Py_None) {
    Py_INCREF(Py_None);
    shp = Py_None;
  } else {
    shp = PySequence_Tuple(v);
    if (!shp) return -1;
  }
  Py_SETREF(self->shape, shp);
  return 0;
}

static PyObject* tensor_repr(TensorObject* self) {
  PyObject* dt = tensor_get_dtype(self, NULL);
  if (!dt) return NULL;
  PyObject* sh = tensor_get_shape(self, NULL);
  if (!sh) {
    Py_DECREF(dt);
    return NULL;
  }
  PyObject* lst = PySequence_List(sh);
  Py_DECREF(sh);
  if (!lst) {
    Py_DECREF(dt);
    return NULL;
  }
  PyObject* r = PyUnicode_FromFormat("Tensor(id=%llu, %S%R)", self->tid, dt, lst);
  Py_DECREF(dt);
  Py_DECREF(lst);
  return r;
}

static PyMemberDef tensor_members[] = {
    {"ctx", T_OBJECT_EX, offsetof(TensorObject, ctx), 0, "the Context (None once released by hand)"},
    {"tid", T_ULONGLONG, offsetof(TensorObject, tid), READONLY, "unique tensor id"},
    {"_dtype", T_OBJECT_EX, offsetof(TensorObject, dtype), 0, "element type name, or None: not asked yet"},
    {"_shape", T_OBJECT_EX, offsetof(TensorObject, shape), 0, "shape tuple, or None: not asked yet"},
    {"_keep", T_OBJECT_EX, offsetof(TensorObject, keep), 0, "owner of the device buffer"},
    {NULL}};

static PyGetSetDef tensor_getset[] = {
    {"dtype", (getter)tensor_get_dtype, (setter)tensor_set_dtype, "element type name", NULL},
    {"shape", (getter)tensor_get_shape, (setter)tensor_set_shape, "shape tuple", NULL},
    {NULL}};

static PyTypeObject TensorType = {
    PyVarObject_HEAD_INIT(NULL, 0)
    .tp_name = "paper_2102_13267_amd._ltrec.Tensor",
    .tp_basicsize = sizeof(TensorObject),
    .tp_dealloc = (destructor)tensor_dealloc,
    .tp_repr = (reprfunc)tensor_repr,
    .tp_flags = Py_TPFLAGS_DEFAULT,
    .tp_doc = "Tensor(ctx, tid, dtype=None, shape=None, keep=None): a handle (unique tensor id)",
    .tp_weaklistoffset = offsetof(TensorObject, weakrefs),
    .tp_members = tensor_members,
    .tp_getset = tensor_getset,
    .tp_new = tensor_new,
};

static PyObject* rec_init(PyObject* self, PyObject* args) {
  unsigned long long a, b, c, d, e, f, g;
  if (!PyArg_ParseTuple(args, "KKKKKKK", &a, &b, &c, &d, &e, &f, &g)) return NULL;
  p_op = (lt_op_fn)(uintptr_t)a;
  p_scalar = (lt_scalar_fn)(uintptr_t)b;
  p_release = (lt_release_fn)(uintptr_t)c;
  p_last_error = (lt_last_error_fn)(uintptr_t)d;
  p_assign = (lt_assign_fn)(uintptr_t)e;
  p_release_many = (lt_release_many_fn)(uintptr_t)f;
  p_barrier = (lt_barrier_fn)(uintptr_t)g;
  Py_RETURN_NONE;
}

/* set_error(cls): raise cls(status, message) instead of _ltrec.Error(status, message) */
static PyObject* rec_set_error(PyObject* self, PyObject* cls) {
  if (!PyExceptionClass_Check(cls)) {
    PyErr_SetString(PyExc_TypeError, "set_error(cls): an exception class");
    return NULL;
  }
  Py_INCREF(cls);
  Py_XSETREF(rec_error, cls);
  Py_RETURN_NONE;
}

static PyObject* rec_set_query(PyObject* self, PyObject* fn) {
  Py_INCREF(fn);
  Py_XSETREF(query_hook, fn);
  Py_RETURN_NONE;
}

static PyObject* raise_status(void* ctx, int st) {
  const char* msg = p_last_error ? p_last_error(ctx) : "";
  PyObject* v = Py_BuildValue("(is)", st, msg ? msg : "");
  if (v) {
    PyErr_SetObject(rec_error, v);
    Py_DECREF(v);
  }
  return NULL;
}

/* Record one op on `items` (tensors or numbers): lt_scalar for the numbers, lt_op, lt_release of
 * those temporaries.  Returns the result tensor (n_out == 1) or a tuple of them. */
static PyObject* record_core(PyObject* owner, void* ctx, long opcode, PyObject* const* items, Py_ssize_t n_in,
                             const void* attrs, long n_attr, long n_out) {
  if (!p_op) {
    PyErr_SetString(PyExc_RuntimeError, "_ltrec.init has not been called");
    return NULL;
  }
  if (n_in > kMaxIn || n_out < 1 || n_out > kMaxOut) {
    PyErr_SetString(PyExc_ValueError, "too many operands or results");
    return NULL;
  }
  uint64_t ids[kMaxIn], temps[kMaxIn], outs[kMaxOut];
  int n_temp = 0, st = 0;
  for (Py_ssize_t i = 0; i < n_in && st == 0; ++i) {
    PyObject* x = items[i];   /* borrowed */
    if (Py_TYPE(x) == &TensorType) {
      ids[i] = ((TensorObject*)x)->tid;
    } else if (PyFloat_Check(x) || PyLong_Check(x)) {
      /* a Python number: a rank-0 fp32 scalar tensor that lives until the op is recorded */
      const double v = PyFloat_Check(x) ? PyFloat_AS_DOUBLE(x) : PyLong_AsDouble(x);
      if (v == -1.0 && PyErr_Occurred()) break;
      st = p_scalar(ctx, 0 /* LT_F32 */, v, &ids[i]);
      if (st == 0) temps[n_temp++] = ids[i];
    } else {
      PyObject* tid = PyObject_GetAttr(x, str_tid);
      if (tid) {
        ids[i] = PyLong_AsUnsignedLongLong(tid);
        Py_DECREF(tid);
        if (PyErr_Occurred()) break;
      } else {
        /* not a tensor: anything else that converts to a float (a NumPy scalar, say) */
        PyErr_Clear();
        const double v = PyFloat_AsDouble(x);
        if (v == -1.0 && PyErr_Occurred()) break;
        st = p_scalar(ctx, 0 /* LT_F32 */, v, &ids[i]);
        if (st == 0) temps[n_temp++] = ids[i];
      }
    }
  }
  if (st == 0 && !PyErr_Occurred()) st = p_op(ctx, (uint16_t)opcode, ids, (int)n_in, attrs, (int)n_attr, outs, (int)n_out);
  for (int t = 0; t < n_temp; ++t) (void)p_release(ctx, temps[t]);
  if (PyErr_Occurred()) return NULL;
  if (st != 0) return raise_status(ctx, st);
  if (n_out == 1) return tensor_make(owner, outs[0]);
  PyObject* tup = PyTuple_New(n_out);
  if (!tup) return NULL;
  for (long k = 0; k < n_out; ++k) {
    PyObject* v = tensor_make(owner, outs[k]);
    if (!v) {
      Py_DECREF(tup);
      return NULL;
    }
    PyTuple_SET_ITEM(tup, k, v);
  }
  return tup;
}

/* op(owner: Context, ctx: int, opcode: int, inputs: sequence of (Tensor | int | float),
 *    attrs_addr: int, n_attr: int, n_out: int) -> Tensor (n_out == 1) or tuple of Tensors */
static PyObject* rec_op(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
  if (nargs != 7) {
    PyErr_SetString(PyExc_TypeError, "op(owner, ctx, opcode, inputs, attrs_addr, n_attr, n_out)");
    return NULL;
  }
  PyObject* owner = args[0];
  void* ctx = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[1]);
  const long opcode = PyLong_AsLong(args[2]);
  const void* attrs = (const void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[4]);
  const long n_attr = PyLong_AsLong(args[5]);
  const long n_out = PyLong_AsLong(args[6]);
  if (PyErr_Occurred()) return NULL;
  PyObject* seq = PySequence_Fast(args[3], "inputs must be a sequence");
  if (!seq) return NULL;
  PyObject* r = record_core(owner, ctx, opcode, PySequence_Fast_ITEMS(seq), PySequence_Fast_GET_SIZE(seq), attrs, n_attr, n_out);
  Py_DECREF(seq);
  return r;
}

/* ---- methods of the binding's Context for ops without attributes ----------------------------
 * PlainOp(name, opcode, min_operands, max_operands, keyword=None) is a method descriptor: stored
 * in the class, `ctx.mul(a, b)` calls it with (ctx, a, b) and no Python frame in between.  The
 * context's handle is its `_hv` attribute.  `keyword` names an optional last operand that may also
 * be passed by keyword, None meaning absent (add's alpha). */
typedef struct {
  PyObject_HEAD
  vectorcallfunc vectorcall;
  long opcode;
  Py_ssize_t min_ops, max_ops;
  PyObject* name;
  PyObject* keyword;   /* interned str or NULL */
} PlainOpObject;

static PyObject* str_hv;

static PyObject* plainop_call(PyObject* callable, PyObject* const* args, size_t nargsf, PyObject* kwnames) {
  PlainOpObject* op = (PlainOpObject*)callable;
  const Py_ssize_t nargs = PyVectorcall_NARGS(nargsf);
  const Py_ssize_t nkw = kwnames ? PyTuple_GET_SIZE(kwnames) : 0;
  if (nargs < 1) {
    PyErr_Format(PyExc_TypeError, "%U() needs the context it is a method of", op->name);
    return NULL;
  }
  PyObject* items[kMaxIn];
  Py_ssize_t n = nargs - 1;
  if (n > op->max_ops || n > kMaxIn) {
    PyErr_Format(PyExc_TypeError, "%U() takes at most %zd operands", op->name, op->max_ops);
    return NULL;
  }
  for (Py_ssize_t i = 0; i < n; ++i) items[i] = args[1 + i];
  if (nkw) {
    if (nkw != 1 || !op->keyword || n != op->max_ops - 1 ||
        PyUnicode_Compare(PyTuple_GET_ITEM(kwnames, 0), op->keyword) != 0) {
      PyErr_Format(PyExc_TypeError, "%U() got an unexpected keyword argument", op->name);
      return NULL;
    }
    items[n++] = args[nargs];
  }
  if (op->keyword && n == op->max_ops && items[n - 1] == Py_None) --n;   /* the optional operand left out */
  if (n < op->min_ops) {
    PyErr_Format(PyExc_TypeError, "%U() takes at least %zd operands", op->name, op->min_ops);
    return NULL;
  }
  PyObject* h = PyObject_GetAttr(args[0], str_hv);
  if (!h) return NULL;
  void* ctx = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(h);
  Py_DECREF(h);
  if (PyErr_Occurred()) return NULL;
  return record_core(args[0], ctx, op->opcode, items, n, NULL, 0, 1);
}

static PyObject* plainop_new(PyTypeObject* type, PyObject* args, PyObject* kw) {
  static char* names[] = {"name", "opcode", "min_operands", "max_operands", "keyword", NULL};
  PyObject *name, *keyword = Py_None;
  long opcode;
  Py_ssize_t lo, hi;
  if (!PyArg_ParseTupleAndKeywords(args, kw, "Ulnn|O", names, &name, &opcode, &lo, &hi, &keyword)) return NULL;
  if (lo < 1 || hi < lo || hi > kMaxIn || (keyword != Py_None && !PyUnicode_Check(keyword))) {
    PyErr_SetString(PyExc_ValueError, "PlainOp(name, opcode, min_operands, max_operands, keyword=None)");
    return NULL;
  }
  PlainOpObject* op = (PlainOpObject*)type->tp_alloc(type, 0);
  if (!op) return NULL;
  op->vectorcall = plainop_call;
  op->opcode = opcode;
  op->min_ops = lo;
  op->max_ops = hi;
  Py_INCREF(name);
  op->name = name;
  if (keyword != Py_None) {
    Py_INCREF(keyword);
    PyUnicode_InternInPlace(&keyword);
    op->keyword = keyword;
  } else {
    op->keyword = NULL;
  }
  return (PyObject*)op;
}

static void plainop_dealloc(PlainOpObject* op) {
  Py_XDECREF(op->name);
  Py_XDECREF(op->keyword);
  Py_TYPE(op)->tp_free((PyObject*)op);
}

static PyObject* plainop_get(PyObject* self, PyObject* obj, PyObject* type) {
  if (!obj || obj == Py_None) {
    Py_INCREF(self);
    return self;
  }
  return PyMethod_New(self, obj);
}

static PyObject* plainop_repr(PlainOpObject* op) { return PyUnicode_FromFormat("<lt op %U (opcode %ld)>", op->name, op->opcode); }

static PyMemberDef plainop_members[] = {
    {"__name__", T_OBJECT_EX, offsetof(PlainOpObject, name), READONLY, "op name"},
    {"opcode", T_LONG, offsetof(PlainOpObject, opcode), READONLY, "opcode recorded"},
    {NULL}};

static PyTypeObject PlainOpType = {
    PyVarObject_HEAD_INIT(NULL, 0)
    .tp_name = "paper_2102_13267_amd._ltrec.PlainOp",
    .tp_basicsize = sizeof(PlainOpObject),
    .tp_dealloc = (destructor)plainop_dealloc,
    .tp_vectorcall_offset = offsetof(PlainOpObject, vectorcall),
    .tp_repr = (reprfunc)plainop_repr,
    .tp_call = PyVectorcall_Call,
    .tp_flags = Py_TPFLAGS_DEFAULT | Py_TPFLAGS_HAVE_VECTORCALL | Py_TPFLAGS_METHOD_DESCRIPTOR,
    .tp_doc = "PlainOp(name, opcode, min_operands, max_operands, keyword=None): a Context method that records one op",
    .tp_members = plainop_members,
    .tp_descr_get = plainop_get,
    .tp_new = plainop_new,
};

/* assign(ctx: int, dst: Tensor, src: Tensor): lt_assign; what is known of src's type and shape
 * becomes what is known of dst's (unknown stays unknown: asked for on demand) */
static PyObject* rec_assign(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
  if (nargs != 3 || Py_TYPE(args[1]) != &TensorType || Py_TYPE(args[2]) != &TensorType) {
    PyErr_SetString(PyExc_TypeError, "assign(ctx, dst: Tensor, src: Tensor)");
    return NULL;
  }
  if (!p_assign) {
    PyErr_SetString(PyExc_RuntimeError, "_ltrec.init has not been called");
    return NULL;
  }
  void* ctx = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[0]);
  if (PyErr_Occurred()) return NULL;
  TensorObject *dst = (TensorObject*)args[1], *src = (TensorObject*)args[2];
  const int st = p_assign(ctx, dst->tid, src->tid);
  if (st != 0) return raise_status(ctx, st);
  Py_INCREF(src->dtype); Py_SETREF(dst->dtype, src->dtype);
  Py_INCREF(src->shape); Py_SETREF(dst->shape, src->shape);
  Py_RETURN_NONE;
}

/* lt_release_many over the ids in the list, which is emptied.  0, or -1 with an exception set. */
static int release_list(void* ctx, PyObject* lst) {
  const Py_ssize_t n = PyList_GET_SIZE(lst);
  if (n == 0) return 0;
  uint64_t* ids = (uint64_t*)PyMem_Malloc((size_t)n * sizeof(uint64_t));
  if (!ids) {
    PyErr_NoMemory();
    return -1;
  }
  for (Py_ssize_t i = 0; i < n; ++i) {
    ids[i] = PyLong_AsUnsignedLongLong(PyList_GET_ITEM(lst, i));
    if (PyErr_Occurred()) {
      PyMem_Free(ids);
      return -1;
    }
  }
  /* (nothing below runs Python code, so no handle can die and grow the list in between) */
  if (PyList_SetSlice(lst, 0, n, NULL) < 0) {
    PyMem_Free(ids);
    return -1;
  }
  if (ctx) (void)p_release_many(ctx, ids, (size_t)n);   /* an id the library no longer knows is not the caller's error */
  PyMem_Free(ids);
  return 0;
}

/* release_many(ctx: int, ids: list of int): lt_release_many over the list, which is emptied */
static PyObject* rec_release_many(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
  if (nargs != 2 || !PyList_Check(args[1])) {
    PyErr_SetString(PyExc_TypeError, "release_many(ctx, ids: list)");
    return NULL;
  }
  if (!p_release_many) {
    PyErr_SetString(PyExc_RuntimeError, "_ltrec.init has not been called");
    return NULL;
  }
  void* ctx = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[0]);
  if (PyErr_Occurred()) return NULL;
  if (release_list(ctx, args[1]) < 0) return NULL;
  Py_RETURN_NONE;
}

/* barrier(ctx: int, dead: list of int, blocking: int, info_addr: int): hands the dropped tensors over
 * (lt_release_many, the list is emptied), then lt_barrier into the lt_barrier_info at info_addr.  The
 * interpreter lock is released while the barrier runs (a blocking one waits for the device). */
static PyObject* rec_barrier(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
  if (nargs != 4 || !PyList_Check(args[1])) {
    PyErr_SetString(PyExc_TypeError, "barrier(ctx, dead: list, blocking, info_addr)");
    return NULL;
  }
  if (!p_barrier || !p_release_many) {
    PyErr_SetString(PyExc_RuntimeError, "_ltrec.init has not been called");
    return NULL;
  }
  void* ctx = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[0]);
  const long blocking = PyLong_AsLong(args[2]);
  void* info = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[3]);
  if (PyErr_Occurred()) return NULL;
  if (release_list(ctx, args[1]) < 0) return NULL;
  int st;
  Py_BEGIN_ALLOW_THREADS
  st = p_barrier(ctx, blocking ? 1 : 0, info);
  Py_END_ALLOW_THREADS
  if (st != 0) return raise_status(ctx, st);
  Py_RETURN_NONE;
}

static PyMethodDef methods[] = {
    {"init", rec_init, METH_VARARGS, "init(lt_op, lt_scalar, lt_release, lt_last_error, lt_assign, lt_release_many, lt_barrier): addresses of the entry points"},
    {"set_error", rec_set_error, METH_O, "set_error(cls): the exception class raised as cls(status, message)"},
    {"set_query", rec_set_query, METH_O, "set_query(fn): fn(tensor) fills in tensor._dtype and tensor._shape"},
    {"op", (PyCFunction)(void (*)(void))rec_op, METH_FASTCALL, "record one op; returns its result tensor(s)"},
    {"assign", (PyCFunction)(void (*)(void))rec_assign, METH_FASTCALL, "record dst <- src"},
    {"release_many", (PyCFunction)(void (*)(void))rec_release_many, METH_FASTCALL, "release the listed tensor ids and empty the list"},
    {"barrier", (PyCFunction)(void (*)(void))rec_barrier, METH_FASTCALL, "release the listed tensor ids, then lt_barrier"},
    {NULL, NULL, 0, NULL}};

static struct PyModuleDef moduledef = {PyModuleDef_HEAD_INIT, "_ltrec", "recording fast path of the lt binding", -1, methods};

PyMODINIT_FUNC PyInit__ltrec(void) {
  PyObject* m = PyModule_Create(&moduledef);
  if (!m) return NULL;
  str_tid = PyUnicode_InternFromString("tid");
  str_dead = PyUnicode_InternFromString("_dead");
  str_kept = PyUnicode_InternFromString("_kept");
  str_hv = PyUnicode_InternFromString("_hv");
  rec_error = PyErr_NewException("_ltrec.Error", NULL, NULL);
  if (!str_tid || !str_dead || !str_kept || !str_hv || !rec_error) return NULL;
  Py_INCREF(rec_error);   /* one reference is the module attribute's, one stays with rec_error */
  if (PyModule_AddObject(m, "Error", rec_error) < 0) return NULL;
  if (PyModule_AddIntConstant(m, "API", 6) < 0) return NULL;   /* bumped when the binding's expectations change */
  if (PyType_Ready(&TensorType) < 0) return NULL;
  Py_INCREF(&TensorType);
  if (PyModule_AddObject(m, "Tensor", (PyObject*)&TensorType) < 0) return NULL;
  if (PyType_Ready(&PlainOpType) < 0) return NULL;
  Py_INCREF(&PlainOpType);
  if (PyModule_AddObject(m, "PlainOp", (PyObject*)&PlainOpType) < 0) return NULL;
  return m;
}
