"""ctypes loader for libevo_gfx950.so (the C ABI declared in include/evo.h).

There is no fallback: if the library has not been built, importing the binding's functions
raises with the build command."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libevo_gfx950.so")

EVO_MAX_LAYERS = 8
EVO_POP_MAX = 4096


class pgpe_config(C.Structure):
    _fields_ = [("P", C.c_int32), ("pop_max", C.c_int32), ("sigma_init", C.c_float), ("lr_mu", C.c_float),
                ("lr_sigma", C.c_float), ("sigma_max_change", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("sigma_rule", C.c_int32), ("shaping", C.c_int32),
                ("optimizer", C.c_int32), ("momentum", C.c_float), ("max_speed", C.c_float)]


class policy_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_layers", C.c_int32), ("dims", C.c_int32 * (EVO_MAX_LAYERS + 1)),
                ("act", C.c_int32 * EVO_MAX_LAYERS), ("dtype", C.c_int32)]


class task_desc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("n_rollouts", C.c_int32), ("B", C.c_int32), ("P", C.c_int32),
                ("reset_seed", C.c_uint64), ("generation", C.c_uint32), ("seq_in", C.c_int32),
                ("obs_dev", C.c_void_p), ("obs_member_stride", C.c_int64), ("target_dev", C.c_void_p),
                ("cp", C.c_float * 8), ("init_scale", C.c_float), ("seq_out", C.c_int32),
                ("work_dev", C.c_void_p), ("generation_dev", C.c_void_p)]


_SIGNATURES = {
    "pgpe_workspace_bytes": (C.c_size_t, [C.POINTER(pgpe_config)]),
    "pgpe_config_defaults": (C.c_int, [C.POINTER(pgpe_config), C.c_int32, C.c_int32]),
    "pgpe_clipup_default_max_speed": (C.c_float, [C.c_float]),
    "pgpe_create": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(pgpe_config), C.c_void_p, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_void_p, C.c_void_p]),
    "pgpe_destroy": (C.c_int, [C.c_void_p]),
    "pgpe_reset": (C.c_int, [C.c_void_p, C.c_void_p]),
    "pgpe_get_generation": (C.c_int, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "pgpe_set_generation": (C.c_int, [C.c_void_p, C.c_uint32]),
    "pgpe_center": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]),
    "pgpe_state_bytes": (C.c_size_t, [C.c_void_p]),
    "pgpe_state_export": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "pgpe_state_import": (C.c_int, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "evo_forage_step": (C.c_int, [C.POINTER(task_desc), C.c_int32] + [C.c_void_p] * 10),
    "evo_forage_state": (C.c_int, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_void_p, C.c_int32, C.c_int32]
                         + [C.c_void_p] * 5),
    "pgpe_device_generation": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_void_p]),
    "pgpe_sync_generation": (C.c_int, [C.c_void_p, C.c_void_p]),
    "pgpe_ask": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]),
    "pgpe_tell": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "pgpe_ask_sphere_workspace_bytes": (C.c_size_t, [C.POINTER(pgpe_config)]),
    "pgpe_ask_sphere": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "pgpe_ask_rollout": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int32, C.POINTER(task_desc), C.POINTER(policy_desc),
                                   C.c_void_p, C.c_void_p]),
    "pgpe_generation": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int32, C.POINTER(task_desc), C.POINTER(policy_desc),
                                  C.c_void_p, C.c_void_p]),
    "evo_ask_forward": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int32, C.POINTER(policy_desc), C.c_void_p, C.c_int64,
                                  C.c_void_p, C.c_int32, C.c_void_p]),
    "pgpe_tell_stored": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "policy_param_count": (C.c_int64, [C.POINTER(policy_desc)]),
    "pop_forward": (C.c_int, [C.POINTER(policy_desc), C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                              C.c_int32, C.c_void_p]),
    "rollout_workspace_bytes": (C.c_size_t, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_int32]),
    "rollout": (C.c_int, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_void_p, C.c_int32, C.c_int32,
                          C.c_void_p, C.c_void_p]),
    "rollout_static_scratch_bytes": (C.c_size_t, []),
    "rollout_static_scratch": (C.c_int, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_void_p, C.c_int32,
                                         C.c_int32, C.c_void_p, C.c_void_p]),
    "evo_philox_u32": (C.c_int, [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                 C.c_void_p, C.c_void_p]),
    "evo_philox_normal": (C.c_int, [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                    C.c_void_p, C.c_void_p]),
    "evo_centered_rank": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "evo_pgpe_gradients": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "evo_task_step": (C.c_int, [C.POINTER(task_desc), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                C.c_void_p]),
    "evo_rollout_details": (C.c_int, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_void_p, C.c_int32,
                                      C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "evo_rollout_trace": (C.c_int, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_void_p, C.c_int32,
                                    C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "evo_seq2seq_logits": (C.c_int, [C.POINTER(task_desc), C.POINTER(policy_desc), C.c_void_p, C.c_int32,
                                     C.c_void_p, C.c_void_p]),
    "evo_probe_rate": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_double), C.c_void_p, C.c_void_p]),
    "evo_last_error": (C.c_char_p, []),
    "evo_version": (C.c_char_p, []),
}

EXPORTS = tuple(_SIGNATURES)
_lib = None


def load():
    """Load the shared library (once) and set the argument types of every export."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2202_05008_amd.build` "
                           "(there is no CPU fallback)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)       # AttributeError if the library does not export it
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib
