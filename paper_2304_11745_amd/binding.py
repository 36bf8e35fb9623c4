"""ctypes binding of include/gacer.h -- same names, argument marshalling only.

The shared library must have been built (``python -m paper_2304_11745_amd.build`` or
``__graft_entry__.build()``); importing this module without it raises.
"""
import ctypes as C
import os

# The library runs on streams and memory that PyTorch creates, so both must use ONE HIP runtime in the
# process: import torch first, then libgacer.so binds to the runtime torch has already loaded.
import torch  # noqa: F401  (load order matters)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgacer.so")

GACER_OK, GACER_EINVAL, GACER_ESHAPE, GACER_EPLAN, GACER_ESTATE, GACER_ENOMEM, GACER_EHIP = range(7)
GACER_F32, GACER_BF16 = 0, 1
(GACER_CONV2D, GACER_DWCONV2D, GACER_GEMM, GACER_BGEMM_QK, GACER_BGEMM_PV, GACER_MAXPOOL, GACER_GAVGPOOL,
 GACER_AFFINE_ACT, GACER_ADD, GACER_LAYERNORM, GACER_SOFTMAX, GACER_ACT, GACER_SCALE, GACER_CONCAT, GACER_AVGPOOL) = range(15)
GACER_ACT_NONE, GACER_ACT_RELU, GACER_ACT_RELU6, GACER_ACT_GELU, GACER_ACT_HSWISH, GACER_ACT_HSIGMOID = range(6)
GACER_AXIS_NONE, GACER_AXIS_BATCH, GACER_AXIS_COUT = range(3)
GACER_MODE_PLAN, GACER_MODE_SEQUENTIAL, GACER_MODE_STREAM_PARALLEL = range(3)

EXPORTS = ["gacer_create", "gacer_destroy", "gacer_load_tenants", "gacer_set_plan", "gacer_plan_from_pointers",
           "gacer_run", "gacer_profile", "gacer_search", "gacer_model_residue", "gacer_plan_free",
           "gacer_last_error", "gacer_launch_count", "gacer_trace_run", "gacer_issue_stats", "gacer_capture",
           "gacer_release_graphs", "gacer_set_issue_threads", "gacer_set_sync_every_launch", "gacer_set_fuse_affine", "gacer_probe_stream_queues", "gacer_place_streams",
           "gacer_refine", "gacer_run_static", "gacer_plan_to_text",
           "gacer_plan_from_text"]


class gacer_tensor(C.Structure):
    _fields_ = [("n", C.c_int64), ("c", C.c_int64), ("h", C.c_int64), ("w", C.c_int64), ("dptr", C.c_void_p),
                ("pitch", C.c_int64), ("base", C.c_int), ("c_off", C.c_int)]


class gacer_op(C.Structure):
    _fields_ = [("kind", C.c_int), ("in0", C.c_int), ("in1", C.c_int), ("res", C.c_int), ("out", C.c_int),
                ("w", C.c_void_p), ("bias", C.c_void_p), ("scale", C.c_void_p), ("shift", C.c_void_p),
                ("cin", C.c_int), ("cout", C.c_int), ("kh", C.c_int), ("kw", C.c_int), ("stride", C.c_int),
                ("pad", C.c_int), ("groups", C.c_int), ("act", C.c_int), ("alpha", C.c_float)]


class gacer_tenant(C.Structure):
    _fields_ = [("n_ops", C.c_int), ("ops", C.POINTER(gacer_op)), ("n_tensors", C.c_int),
                ("tensors", C.POINTER(gacer_tensor)), ("input", C.c_int), ("output", C.c_int),
                ("dtype", C.c_int), ("batch", C.c_int), ("stream", C.c_void_p), ("sibling_stream", C.c_void_p)]


class gacer_split(C.Structure):
    _fields_ = [("tenant", C.c_int), ("op", C.c_int), ("axis", C.c_int), ("factor", C.c_int), ("sizes", C.POINTER(C.c_int)),
                ("sibling", C.c_int)]


class gacer_sync(C.Structure):
    _fields_ = [("src_tenant", C.c_int), ("src_op", C.c_int), ("dst_tenant", C.c_int), ("dst_op", C.c_int),
                ("when", C.c_int)]


class gacer_plan(C.Structure):
    _fields_ = [("n_split", C.c_int), ("split", C.POINTER(gacer_split)), ("n_sync", C.c_int),
                ("sync", C.POINTER(gacer_sync))]


class gacer_prof(C.Structure):
    _fields_ = [("tenant", C.c_int), ("op", C.c_int), ("axis", C.c_int), ("factor", C.c_int), ("ms", C.c_float),
                ("workgroups", C.c_int), ("cu_share", C.c_float), ("bw_share", C.c_float)]


class gacer_launch_stat(C.Structure):
    _fields_ = [("tenant", C.c_int), ("op", C.c_int), ("chunk", C.c_int), ("ms", C.c_float), ("flops", C.c_double),
                ("bytes", C.c_double), ("workgroups", C.c_int), ("kernel", C.c_char * 40), ("start_ms", C.c_float),
                ("end_ms", C.c_float)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2304_11745_amd.build); "
                          "there is no fallback implementation")
    lib = C.CDLL(LIB_PATH)
    ctx = C.c_void_p
    lib.gacer_create.argtypes = [C.POINTER(ctx)]
    lib.gacer_destroy.argtypes = [ctx]
    lib.gacer_destroy.restype = None
    lib.gacer_load_tenants.argtypes = [ctx, C.POINTER(gacer_tenant), C.c_int]
    lib.gacer_set_plan.argtypes = [ctx, C.POINTER(gacer_plan)]
    lib.gacer_plan_from_pointers.argtypes = [ctx, C.POINTER(C.c_int), C.c_int, C.POINTER(C.POINTER(gacer_plan))]
    lib.gacer_run.argtypes = [ctx, C.c_int, C.c_int, C.POINTER(C.c_float)]
    lib.gacer_run_static.argtypes = [ctx, C.c_int, C.c_int]
    lib.gacer_profile.argtypes = [ctx, C.POINTER(gacer_prof), C.c_size_t, C.POINTER(C.c_size_t)]
    lib.gacer_search.argtypes = [ctx, C.POINTER(gacer_prof), C.c_size_t, C.c_int, C.POINTER(C.POINTER(gacer_plan)),
                                 C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_double)]
    lib.gacer_model_residue.argtypes = [ctx, C.POINTER(gacer_prof), C.c_size_t, C.POINTER(gacer_split), C.c_int,
                                        C.POINTER(C.c_int), C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.gacer_plan_to_text.argtypes = [C.POINTER(gacer_plan), C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)]
    lib.gacer_plan_from_text.argtypes = [C.c_char_p, C.POINTER(C.POINTER(gacer_plan))]
    lib.gacer_plan_free.argtypes = [C.POINTER(gacer_plan)]
    lib.gacer_plan_free.restype = None
    lib.gacer_last_error.argtypes = [ctx]
    lib.gacer_last_error.restype = C.c_char_p
    lib.gacer_launch_count.argtypes = [ctx, C.c_int, C.POINTER(C.c_int)]
    lib.gacer_trace_run.argtypes = [ctx, C.c_int, C.c_int, C.POINTER(gacer_launch_stat), C.c_size_t, C.POINTER(C.c_size_t)]
    lib.gacer_capture.argtypes = [ctx, C.c_int]
    lib.gacer_set_issue_threads.argtypes = [ctx, C.c_int]
    lib.gacer_set_sync_every_launch.argtypes = [ctx, C.c_int]
    lib.gacer_set_fuse_affine.argtypes = [ctx, C.c_int]
    lib.gacer_release_graphs.argtypes = [ctx]
    lib.gacer_issue_stats.argtypes = [ctx, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.gacer_probe_stream_queues.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.POINTER(C.c_int)]
    lib.gacer_place_streams.argtypes = [C.POINTER(gacer_tenant), C.c_int, C.POINTER(C.c_void_p), C.c_int, C.POINTER(C.c_int),
                                        C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.gacer_refine.argtypes = [ctx, C.POINTER(gacer_prof), C.c_size_t, C.c_int, C.c_float, C.POINTER(C.POINTER(gacer_plan)),
                                 C.POINTER(C.c_float)]
    return lib


lib = _load()

gacer_create = lib.gacer_create
gacer_destroy = lib.gacer_destroy
gacer_load_tenants = lib.gacer_load_tenants
gacer_set_plan = lib.gacer_set_plan
gacer_plan_from_pointers = lib.gacer_plan_from_pointers
gacer_run = lib.gacer_run
gacer_run_static = lib.gacer_run_static
gacer_profile = lib.gacer_profile
gacer_search = lib.gacer_search
gacer_model_residue = lib.gacer_model_residue
gacer_plan_free = lib.gacer_plan_free
gacer_plan_to_text = lib.gacer_plan_to_text
gacer_plan_from_text = lib.gacer_plan_from_text
gacer_last_error = lib.gacer_last_error
gacer_launch_count = lib.gacer_launch_count
gacer_trace_run = lib.gacer_trace_run
gacer_issue_stats = lib.gacer_issue_stats
gacer_capture = lib.gacer_capture
gacer_set_issue_threads = lib.gacer_set_issue_threads
gacer_set_sync_every_launch = lib.gacer_set_sync_every_launch
gacer_set_fuse_affine = lib.gacer_set_fuse_affine
gacer_release_graphs = lib.gacer_release_graphs
gacer_probe_stream_queues = lib.gacer_probe_stream_queues
gacer_place_streams = lib.gacer_place_streams
gacer_refine = lib.gacer_refine


class GacerError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"gacer status {status}: {text}")
        self.status = status


def check(ctx, status):
    if status != GACER_OK:
        raise GacerError(status, gacer_last_error(ctx).decode())
