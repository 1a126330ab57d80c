"""ctypes prototypes of the C boundary declared in include/haflo.h.

Argument marshalling only: this module declares argument and result types for
every exported entry point and holds no arithmetic.
"""
import ctypes as C

c_void_p = C.c_void_p
c_size_t = C.c_size_t
c_int = C.c_int
c_u32 = C.c_uint32
c_u64 = C.c_uint64
c_i64 = C.c_int64

# name -> (restype, argtypes)
PROTOTYPES = {
    "haflo_strerror": (C.c_char_p, [c_int]),
    "haflo_keygen": (c_int, [c_u32, c_u64, c_void_p, c_void_p]),
    "haflo_ctx_create_private": (c_int, [c_void_p, c_void_p, c_u32, C.POINTER(c_void_p)]),
    "haflo_ctx_create_public": (c_int, [c_void_p, c_u32, C.POINTER(c_void_p)]),
    "haflo_ctx_destroy": (c_int, [c_void_p]),
    "haflo_ctx_info": (c_int, [c_void_p, C.POINTER(c_u32), C.POINTER(c_u32), C.POINTER(c_u32),
                               C.POINTER(c_size_t), C.POINTER(c_size_t)]),
    "haflo_ctx_set_xtd_bucket_min_rows": (c_int, [c_void_p, c_size_t]),
    "haflo_op_cost": (c_int, [c_void_p, c_int, C.POINTER(c_u64), C.POINTER(c_u32)]),
    "haflo_op_work": (c_int, [c_void_p, c_int, C.POINTER(c_u64)]),
    "haflo_workspace_bytes": (c_size_t, [c_void_p, c_int, c_size_t, c_size_t]),
    "haflo_import_cipher": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_export_cipher": (c_int, [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_encode_f32": (c_int, [c_void_p, c_void_p, c_u32, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_encode_exponents_f32": (c_int, [c_void_p, c_u32, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_decode": (c_int, [c_void_p, c_void_p, c_u32, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_encrypt": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]),
    "haflo_decrypt": (c_int, [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]),
    "haflo_decrypt_static": (c_int, [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_add": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_scalar_mul_u64": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]),
    "haflo_scalar_mul_i64_bcast": (c_int, [c_void_p, c_void_p, c_i64, c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]),
    "haflo_cipher_matvec": (c_int, [c_void_p, c_int, c_void_p, c_void_p, c_size_t, c_size_t, c_void_p, c_void_p,
                                    c_size_t, c_void_p]),
    "haflo_fore_gradient": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_u32, c_void_p, c_void_p, c_size_t,
                                    c_void_p, c_size_t, c_void_p]),
    "haflo_taylor_loss": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_u32, c_void_p, c_void_p,
                                  c_size_t, c_void_p, c_size_t, c_void_p]),
    "haflo_stager_create": (c_int, [c_void_p, c_size_t, c_size_t, C.POINTER(c_void_p)]),
    "haflo_stager_destroy": (c_int, [c_void_p]),
    "haflo_stager_stats": (c_int, [c_void_p, C.POINTER(c_size_t), C.POINTER(c_size_t),
                                   C.POINTER(c_size_t)]),
    "haflo_stage_in_cipher": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_stage_in_plain": (c_int, [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_stage_out_cipher": (c_int, [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_stage_out_plain": (c_int, [c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_encrypt_with_obfuscator": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p, c_size_t,
                                              c_void_p]),
    "haflo_cipher_sum": (c_int, [c_void_p, c_void_p, c_size_t, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_cipher_sum_segments": (c_int, [c_void_p, c_void_p, c_size_t, c_void_p, c_size_t, c_void_p, c_void_p, c_void_p,
                                          c_size_t, c_void_p]),
    "haflo_store_create": (c_int, [c_void_p, c_void_p, c_size_t, c_void_p, C.POINTER(c_void_p)]),
    "haflo_store_destroy": (c_int, [c_void_p]),
    "haflo_store_stats": (c_int, [c_void_p, C.POINTER(c_size_t), C.POINTER(c_size_t), C.POINTER(c_size_t),
                                  C.POINTER(c_size_t)]),
    "haflo_store_new": (c_int, [c_void_p, c_int, c_size_t, c_u32, C.POINTER(c_u64)]),
    "haflo_store_info": (c_int, [c_void_p, c_u64, C.POINTER(c_int), C.POINTER(c_size_t), C.POINTER(c_void_p),
                                 C.POINTER(c_u32)]),
    "haflo_store_release": (c_int, [c_void_p, c_u64]),
    "haflo_h_upload": (c_int, [c_void_p, c_int, c_void_p, c_int, c_size_t, c_u32, C.POINTER(c_u64)]),
    "haflo_h_download": (c_int, [c_void_p, c_u64, c_void_p, c_int]),
    "haflo_h_encode": (c_int, [c_void_p, c_u64, c_u32, c_u32, C.POINTER(c_u64), C.POINTER(c_u64)]),
    "haflo_h_encode_exponents": (c_int, [c_void_p, c_u64, c_u32, c_u32, C.POINTER(c_u64), C.POINTER(c_u64)]),
    "haflo_h_decode": (c_int, [c_void_p, c_u64, c_u32, c_u32, C.POINTER(c_u64), C.POINTER(c_u64)]),
    "haflo_h_encrypt": (c_int, [c_void_p, c_u64, c_u64, c_u32, C.POINTER(c_u64)]),
    "haflo_h_decrypt": (c_int, [c_void_p, c_u64, c_u32, C.POINTER(c_u64)]),
    "haflo_h_add": (c_int, [c_void_p, c_u64, c_u64, c_u32, C.POINTER(c_u64)]),
    "haflo_h_scalar_mul": (c_int, [c_void_p, c_u64, c_i64, c_u32, C.POINTER(c_u64)]),
    "haflo_h_scalar_mul_each": (c_int, [c_void_p, c_u64, c_u64, c_u32, C.POINTER(c_u64)]),
    "haflo_h_matvec": (c_int, [c_void_p, c_int, c_u64, c_u64, c_size_t, c_size_t, c_u32, C.POINTER(c_u64)]),
    "haflo_h_sum": (c_int, [c_void_p, c_u64, c_u32, C.POINTER(c_u64)]),
}

# include/haflo_peak.h (libhaflo_peak.so)
PEAK_PROTOTYPES = {
    "haflo_peak_streams": (c_int, []),
    "haflo_peak_alu": (c_int, [c_int, c_int, c_int, c_void_p, c_void_p]),
    "haflo_peak_hbm": (c_int, [c_int, c_int, c_void_p, c_void_p, c_size_t, c_void_p]),
    "haflo_peak_limbs": (c_int, [c_int, C.POINTER(c_u32), C.POINTER(c_u32)]),
    "haflo_peak_montmul_chain": (c_int, [c_int, c_void_p, c_void_p, c_void_p, c_u64, c_int, c_void_p, c_size_t, c_void_p]),
}
LIMBS_29_MAD64, LIMBS_29_MAD64_SQUARE, LIMBS_24_MUL24, LIMBS_23_FMA64 = 0, 1, 2, 3
PEAK_MAD_U64_U32, PEAK_MUL_LO_HI, PEAK_MUL_U24, PEAK_FMA_F64, PEAK_ADD_U32 = 0, 1, 2, 3, 4
PEAK_FILL, PEAK_COPY, PEAK_READ = 0, 1, 2

KIND_CIPHER, KIND_PLAIN, KIND_F32, KIND_F64, KIND_I32, KIND_U32, KIND_I64, KIND_U64 = 1, 2, 3, 4, 5, 6, 7, 8

OP_ENCRYPT, OP_DECRYPT, OP_SCALAR_MUL, OP_MATVEC_XT_D, OP_MATVEC_X_W, OP_FORE_GRADIENT, OP_TAYLOR_LOSS, OP_ENCRYPT_OBFUSCATOR = 1, 2, 3, 4, 5, 6, 7, 8
OP_SUM_SEGMENTS = 9


def bind(lib, names=None, prototypes=None):
    """Attach the prototypes to a loaded library; raises AttributeError when a
    declared symbol is missing."""
    for name, (res, args) in (PROTOTYPES if prototypes is None else prototypes).items():
        if names is not None and name not in names:
            continue
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib
