/* CPython marshalling for the calls that a backward pass makes once per
 * parameter (Algorithm 1's autograd_hook fires per gradient): ddp_mark_ready,
 * ddp_mark_ready_many, ddp_finalize_backward.  Through ctypes such a call costs
 * about a microsecond of interpreter time, which for a model with hundreds of
 * parameters is as long as the synchronization itself; here it is an integer
 * conversion and an indirect call.  No arithmetic of the method happens here:
 * the functions receive the addresses of the library's C entry points from the
 * Python binding and pass their arguments through.
 */
#define PY_SSIZE_T_CLEAN
#include <Python.h>
#include <stdint.h>

typedef int32_t (*mark_fn)(void*, int32_t);
typedef int32_t (*finalize_fn)(void*);

static mark_fn g_mark = NULL;
static finalize_fn g_finalize = NULL;

static PyObject* bind_entry_points(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
    if (nargs != 2) {
        PyErr_SetString(PyExc_TypeError, "bind(mark_ready_address, finalize_backward_address)");
        return NULL;
    }
    void* a = PyLong_AsVoidPtr(args[0]);
    if (a == NULL && PyErr_Occurred()) return NULL;
    void* b = PyLong_AsVoidPtr(args[1]);
    if (b == NULL && PyErr_Occurred()) return NULL;
    g_mark = (mark_fn)a;
    g_finalize = (finalize_fn)b;
    Py_RETURN_NONE;
}

/* mark_ready(ctx_address, param_id) -> status */
static PyObject* mark_ready(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
    if (nargs != 2 || g_mark == NULL) {
        PyErr_SetString(PyExc_TypeError, "mark_ready(ctx_address, param_id) after bind()");
        return NULL;
    }
    void* ctx = PyLong_AsVoidPtr(args[0]);
    if (ctx == NULL && PyErr_Occurred()) return NULL;
    const long p = PyLong_AsLong(args[1]);
    if (p == -1 && PyErr_Occurred()) return NULL;
    if (p < INT32_MIN || p > INT32_MAX) {
        PyErr_SetString(PyExc_OverflowError, "param_id does not fit int32");
        return NULL;
    }
    return PyLong_FromLong((long)g_mark(ctx, (int32_t)p));
}

/* finalize_backward(ctx_address) -> status */
static PyObject* finalize_backward(PyObject* self, PyObject* const* args, Py_ssize_t nargs) {
    if (nargs != 1 || g_finalize == NULL) {
        PyErr_SetString(PyExc_TypeError, "finalize_backward(ctx_address) after bind()");
        return NULL;
    }
    void* ctx = PyLong_AsVoidPtr(args[0]);
    if (ctx == NULL && PyErr_Occurred()) return NULL;
    return PyLong_FromLong((long)g_finalize(ctx));
}

static PyMethodDef methods[] = {
    {"bind", (PyCFunction)(void (*)(void))bind_entry_points, METH_FASTCALL, "set the C entry points"},
    {"mark_ready", (PyCFunction)(void (*)(void))mark_ready, METH_FASTCALL, "ddp_mark_ready"},
    {"finalize_backward", (PyCFunction)(void (*)(void))finalize_backward, METH_FASTCALL, "ddp_finalize_backward"},
    {NULL, NULL, 0, NULL},
};

static struct PyModuleDef module = {PyModuleDef_HEAD_INIT, "_ddp_fastcall", NULL, -1, methods};

PyMODINIT_FUNC PyInit__ddp_fastcall(void) { return PyModule_Create(&module); }
