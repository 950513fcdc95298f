/* Recording fast path of the Python binding (CPython extension `_ltrec`).
 *
 * Recording an op is the hot path of the method on the host (section 3: every tensor operation of
 * the user's program becomes one call), and a ctypes call costs several times what lt_op itself
 * does.  This module makes the same C-ABI calls -- lt_scalar for Python numbers among the
 * operands, lt_op, lt_release for those temporaries -- from C.  It holds no state of the method
 * and links against nothing: the binding passes the addresses of the four entry points once.
 */
#define PY_SSIZE_T_CLEAN
#include <Python.h>
#include <stdint.h>

typedef int (*lt_op_fn)(void* ctx, uint16_t opcode, const uint64_t* inputs, int n_in, const void* attrs, int n_attr,
                        uint64_t* outputs, int n_out);
typedef int (*lt_scalar_fn)(void* ctx, int dtype, double value, uint64_t* out);
typedef int (*lt_release_fn)(void* ctx, uint64_t t);
typedef const char* (*lt_last_error_fn)(void* ctx);

static lt_op_fn p_op;
static lt_scalar_fn p_scalar;
static lt_release_fn p_release;
static lt_last_error_fn p_last_error;
static PyObject* str_tid;
static PyObject* rec_error;

enum { kMaxIn = 8, kMaxOut = 4 };

static PyObject* rec_init(PyObject* self, PyObject* args) {
  unsigned long long a, b, c, d;
  if (!PyArg_ParseTuple(args, "KKKK", &a, &b, &c, &d)) return NULL;
  p_op = (lt_op_fn)(uintptr_t)a;
  p_scalar = (lt_scalar_fn)(uintptr_t)b;
  p_release = (lt_release_fn)(uintptr_t)c;
  p_last_error = (lt_last_error_fn)(uintptr_t)d;
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

/* op(ctx: int, opcode: int, inputs: sequence of (object with .tid | int | float), attrs_addr: int,
 *    n_attr: int, n_out: int) -> tensor id (n_out == 1) or tuple of ids */
static PyObject* rec_op(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
  if (nargs != 6) {
    PyErr_SetString(PyExc_TypeError, "op(ctx, opcode, inputs, attrs_addr, n_attr, n_out)");
    return NULL;
  }
  if (!p_op) {
    PyErr_SetString(PyExc_RuntimeError, "_ltrec.init has not been called");
    return NULL;
  }
  void* ctx = (void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[0]);
  const long opcode = PyLong_AsLong(args[1]);
  const void* attrs = (const void*)(uintptr_t)PyLong_AsUnsignedLongLong(args[3]);
  const long n_attr = PyLong_AsLong(args[4]);
  const long n_out = PyLong_AsLong(args[5]);
  if (PyErr_Occurred()) return NULL;
  PyObject* seq = PySequence_Fast(args[2], "inputs must be a sequence");
  if (!seq) return NULL;
  const Py_ssize_t n_in = PySequence_Fast_GET_SIZE(seq);
  if (n_in > kMaxIn || n_out < 1 || n_out > kMaxOut) {
    Py_DECREF(seq);
    PyErr_SetString(PyExc_ValueError, "too many operands or results");
    return NULL;
  }
  uint64_t ids[kMaxIn], temps[kMaxIn], outs[kMaxOut];
  int n_temp = 0, st = 0;
  for (Py_ssize_t i = 0; i < n_in && st == 0; ++i) {
    PyObject* x = PySequence_Fast_GET_ITEM(seq, i);   /* borrowed */
    if (PyFloat_Check(x) || PyLong_Check(x)) {
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
  Py_DECREF(seq);
  if (st == 0 && !PyErr_Occurred()) st = p_op(ctx, (uint16_t)opcode, ids, (int)n_in, attrs, (int)n_attr, outs, (int)n_out);
  for (int t = 0; t < n_temp; ++t) (void)p_release(ctx, temps[t]);
  if (PyErr_Occurred()) return NULL;
  if (st != 0) return raise_status(ctx, st);
  if (n_out == 1) return PyLong_FromUnsignedLongLong(outs[0]);
  PyObject* tup = PyTuple_New(n_out);
  if (!tup) return NULL;
  for (long k = 0; k < n_out; ++k) {
    PyObject* v = PyLong_FromUnsignedLongLong(outs[k]);
    if (!v) {
      Py_DECREF(tup);
      return NULL;
    }
    PyTuple_SET_ITEM(tup, k, v);
  }
  return tup;
}

static PyMethodDef methods[] = {
    {"init", rec_init, METH_VARARGS, "init(lt_op, lt_scalar, lt_release, lt_last_error): addresses of the entry points"},
    {"op", (PyCFunction)(void (*)(void))rec_op, METH_FASTCALL, "record one op; returns its tensor id(s)"},
    {NULL, NULL, 0, NULL}};

static struct PyModuleDef moduledef = {PyModuleDef_HEAD_INIT, "_ltrec", "recording fast path of the lt binding", -1, methods};

PyMODINIT_FUNC PyInit__ltrec(void) {
  PyObject* m = PyModule_Create(&moduledef);
  if (!m) return NULL;
  str_tid = PyUnicode_InternFromString("tid");
  rec_error = PyErr_NewException("_ltrec.Error", NULL, NULL);
  if (!str_tid || !rec_error) return NULL;
  Py_INCREF(rec_error);
  if (PyModule_AddObject(m, "Error", rec_error) < 0) return NULL;
  return m;
}
