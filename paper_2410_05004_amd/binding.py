"""ctypes binding with the same names as include/hcache.h (argument marshalling only)."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
# HCACHE_LIB names another build of the library (the diagnostic variants of build.py --diag)
_LIB_FILE = os.environ.get("HCACHE_LIB") or os.path.join(HERE, "libhcache.so")

HC_OK, HC_EINVAL, HC_ERANGE, HC_EALIGN, HC_ENOMEM, HC_EHIP, HC_ESTATE = 0, -1, -2, -3, -4, -5, -6
HC_DEV_BAD_POSITION, HC_DEV_BAD_PAGE = 1, 2
HC_NORM_RMS, HC_NORM_LAYER = 0, 1
_STATUS_NAMES = {0: "HC_OK", -1: "HC_EINVAL", -2: "HC_ERANGE", -3: "HC_EALIGN", -4: "HC_ENOMEM",
                 -5: "HC_EHIP", -6: "HC_ESTATE"}


class HCacheError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


class ModelDesc(C.Structure):
    """Mirror of hc_model_desc."""
    _fields_ = [
        ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
        ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("block_size", C.c_int32),
        ("max_position", C.c_int32), ("rope_style", C.c_int32),
        ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("norm_kind", C.c_int32),
    ]


def lib_path():
    return _LIB_FILE


def _load():
    if not os.path.exists(_LIB_FILE):
        raise ImportError(
            f"{_LIB_FILE} is missing: build it with `python paper_2410_05004_amd/build.py` "
            "(there is no CPU fallback for the restoration path)")
    # The device pointers and stream handles this library is handed come from the caller's HIP
    # runtime, so both must be the same loaded runtime.  PyTorch wheels bundle their own
    # libamdhip64; when PyTorch is installed, load it first so that libhcache.so binds to that
    # copy instead of pulling in a second one.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(_LIB_FILE)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    p = C.POINTER
    sigs = {
        "hc_last_error": (C.c_char_p, []),
        "hc_version": (C.c_char_p, []),
        "hc_validate_desc": (i32, [p(ModelDesc)]),
        "hc_create": (i32, [p(ModelDesc), p(vp)]),
        "hc_destroy": (i32, [vp]),
        "hc_set_layer_weights": (i32, [vp, i32, vp, vp, vp]),
        "hc_set_layer_weights_affine": (i32, [vp, i32, vp, vp, vp, vp, vp]),
        "hc_set_kv_pool": (i32, [vp, i32, vp, i64]),
        "hc_restore_kv": (i32, [vp, i32, vp, vp, i32, vp, i32, vp]),
        "hc_restore_kv_layers": (i32, [vp, i32, i32, p(vp), vp, i32, vp, i32, vp]),
        "hc_restore_kv_ragged": (i32, [vp, i32, vp, vp, i32, vp, i32, vp, i32, vp]),
        "hc_poll_device_error": (i32, [vp, vp, p(i32)]),
        "hc_store_create": (i32, [i32, i32, i32, i64, p(vp)]),
        "hc_store_create_ex": (i32, [i32, i32, i32, i64, i32, p(vp)]),
        "hc_store_destroy": (i32, [vp]),
        "hc_store_append": (i32, [vp, i64, i32, vp, i32]),
        "hc_store_tokens": (i64, [vp, i64, i32]),
        "hc_store_chunk": (i32, [vp, i64, i32, i32, p(vp), p(i32)]),
        "hc_store_drop": (i32, [vp, i64]),
        "hc_restore_context": (i32, [vp, vp, i64, i32, i32, i32, vp, i32, vp, vp]),
        "hc_restore_context_static": (i32, [vp, vp, i64, i32, i32, i32, vp, i32, vp, vp]),
        "hc_static_stage_bytes": (i64, []),
        "hc_poison_staging": (i32, [vp, vp]),
        "hc_gather_kv": (i32, [vp, i32, vp, vp, i32, vp, i32, vp]),
        "hc_scatter_kv": (i32, [vp, i32, vp, vp, i32, vp, i32, vp]),
        "hc_restore_contexts": (i32, [vp, vp, i32, vp, vp, vp, i32, vp, vp]),
        "hc_restore_context_mixed": (i32, [vp, vp, vp, i32, i64, i32, i32, i32, vp, i32, vp, vp]),
        "hc_set_loader": (i32, [vp, i32]),
        "hc_set_split": (i32, [vp, i32]),
        "hc_diag_split_plan": (i32, [i32, i32, i32, i32, p(i32)]),
        "hc_partition_layers": (i32, [i32, C.c_double, C.c_double, C.c_double, C.c_double,
                                      p(i32), p(i32), p(i32)]),
        "hc_saver_create": (i32, [vp, i32, i32, i32, p(vp)]),
        "hc_saver_destroy": (i32, [vp]),
        "hc_saver_save_layer": (i32, [vp, i32, vp, i32, vp, vp, vp]),
        "hc_saver_save_layer_deferred": (i32, [vp, i32, vp, i32, vp, vp, vp]),
        "hc_saver_fence": (i32, [vp, vp]),
        "hc_saver_save_layer_host": (i32, [vp, i32, vp, i32, vp]),
        "hc_saver_flush": (i32, [vp]),
        "hc_diag_tile_map": (i32, [i32, i32, i32, p(i32), p(i32), C.c_int64]),
        "hc_diag_mfma_duty": (i32, [C.c_double, C.c_double, i32, C.c_double, i32, i32, p(C.c_double)]),
        "hc_timing_begin": (i32, [vp]),
        "hc_timing_end": (i32, [vp, vp, p(C.c_double), p(i32)]),
        "hc_timing_end_stats": (i32, [vp, vp, p(C.c_double), p(C.c_double), p(C.c_double), p(i32)]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()
EXPORTED = ("hc_last_error hc_version hc_validate_desc hc_create hc_destroy hc_set_layer_weights "
            "hc_set_kv_pool hc_restore_kv hc_restore_kv_ragged hc_poll_device_error hc_store_create "
            "hc_store_create_ex hc_store_destroy hc_store_append hc_store_tokens hc_store_chunk "
            "hc_store_drop hc_restore_context hc_set_loader hc_timing_begin hc_timing_end "
            "hc_saver_create hc_saver_destroy hc_saver_save_layer hc_saver_save_layer_host "
            "hc_saver_flush hc_partition_layers hc_gather_kv hc_scatter_kv "
            "hc_restore_context_mixed hc_set_layer_weights_affine hc_saver_save_layer_deferred "
            "hc_saver_fence hc_restore_kv_layers hc_restore_contexts hc_timing_end_stats "
            "hc_restore_context_static hc_static_stage_bytes hc_poison_staging hc_diag_mfma_duty hc_diag_tile_map hc_set_split hc_diag_split_plan").split()


def _check(status):
    if status != HC_OK:
        raise HCacheError(status, lib.hc_last_error().decode())


def static_stage_bytes():
    return lib.hc_static_stage_bytes()


def diag_split_plan(d_model, d_kv, n_tok, mode=1):
    """hc_diag_split_plan as a dict."""
    out = (C.c_int32 * 8)()
    _check(lib.hc_diag_split_plan(d_model, d_kv, n_tok, mode, out))
    keys = ("split", "nf", "nt", "nt_main", "n_tail", "n_split", "main_slots", "fixup_workgroups")
    return dict(zip(keys, [int(v) for v in out]))


def diag_tile_map(d_kv, n_tok, n_layers=1):
    """(shape dict, tiles int32 [n_layers, slots, 2]) of a restoration launch; host only."""
    import numpy as np
    shape = (C.c_int32 * 6)()
    _check(lib.hc_diag_tile_map(d_kv, n_tok, n_layers, shape, None, 0))
    slots = shape[4]
    tiles = np.empty((n_layers, slots, 2), dtype=np.int32)
    _check(lib.hc_diag_tile_map(d_kv, n_tok, n_layers, shape,
                                tiles.ctypes.data_as(C.POINTER(C.c_int32)), n_layers * slots))
    return {"nf": shape[0], "nt": shape[1], "gf": shape[2], "gt": shape[3], "slots": slots}, tiles


def diag_mfma_duty(period_us, duty, half_phase=False, total_us=60000.0, zero_operands=False, op_shape=0):
    """Matrix-op rate (TFLOP/s, whole chip) inside the busy windows of a duty-cycled burst."""
    out = C.c_double(0)
    _check(lib.hc_diag_mfma_duty(period_us, duty, 1 if half_phase else 0, total_us,
                                 1 if zero_operands else 0, op_shape, C.byref(out)))
    return out.value


def version():
    return lib.hc_version().decode()


def validate_desc(desc):
    _check(lib.hc_validate_desc(C.byref(desc)))


def partition_layers(n_layers, io_h, io_kv, c_h, c_token):
    """(l_h, l_o, complement) of the bubble-free layer partition; complement 0 = KV offload,
    1 = token recomputation."""
    lh, lo, comp = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(lib.hc_partition_layers(n_layers, io_h, io_kv, c_h, c_token, C.byref(lh), C.byref(lo),
                                   C.byref(comp)))
    return lh.value, lo.value, comp.value


def _ptr(x):
    """Address of a torch tensor / numpy array / int (None -> NULL)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


class Context:
    """Owner of an hc_ctx*.  Methods carry the names of the C entry points."""

    def __init__(self, desc):
        self.desc = desc
        h = C.c_void_p()
        _check(lib.hc_create(C.byref(desc), C.byref(h)))
        self._h = h

    def destroy(self):
        if self._h:
            lib.hc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def set_layer_weights(self, layer, d_wkv, d_gamma, stream=0):
        _check(lib.hc_set_layer_weights(self._h, layer, _ptr(d_wkv), _ptr(d_gamma), stream))

    def set_layer_weights_affine(self, layer, d_wkv, d_gamma, d_beta, d_bias, stream=0):
        _check(lib.hc_set_layer_weights_affine(self._h, layer, _ptr(d_wkv), _ptr(d_gamma),
                                               _ptr(d_beta), _ptr(d_bias), stream))

    def set_kv_pool(self, layer, d_pool, num_pages):
        _check(lib.hc_set_kv_pool(self._h, layer, _ptr(d_pool), num_pages))

    def restore_kv(self, layer, d_hidden, d_positions, n_tok, d_block_table, n_blocks, stream=0):
        _check(lib.hc_restore_kv(self._h, layer, _ptr(d_hidden), _ptr(d_positions), n_tok,
                                 _ptr(d_block_table), n_blocks, stream))

    def restore_kv_layers(self, layer_begin, d_hidden_list, d_positions, n_tok, d_block_table,
                          n_blocks, stream=0):
        """d_hidden_list: one device tensor (or address) per layer, starting at layer_begin."""
        n = len(d_hidden_list)
        arr = (C.c_void_p * max(n, 1))(*[_ptr(h) for h in d_hidden_list])
        _check(lib.hc_restore_kv_layers(self._h, layer_begin, n, arr, _ptr(d_positions), n_tok,
                                        _ptr(d_block_table), n_blocks, stream))

    def restore_kv_ragged(self, layer, d_hidden, d_positions, total_tokens, d_cu_seqlens, n_seq,
                          d_block_tables, max_blocks, stream=0):
        _check(lib.hc_restore_kv_ragged(self._h, layer, _ptr(d_hidden), _ptr(d_positions),
                                        total_tokens, _ptr(d_cu_seqlens), n_seq,
                                        _ptr(d_block_tables), max_blocks, stream))

    def poll_device_error(self, stream=0):
        flags = C.c_int32(0)
        _check(lib.hc_poll_device_error(self._h, stream, C.byref(flags)))
        return flags.value

    def restore_context(self, store, seq_id, tok_begin, n_tok, pos_offset, d_block_table, n_blocks,
                        compute_stream, copy_stream):
        _check(lib.hc_restore_context(self._h, store._h, seq_id, tok_begin, n_tok, pos_offset,
                                      _ptr(d_block_table), n_blocks, compute_stream, copy_stream))

    def poison_staging(self, compute_stream):
        _check(lib.hc_poison_staging(self._h, compute_stream))

    def restore_context_static(self, store, seq_id, tok_begin, n_tok, pos_offset, d_block_table,
                               n_blocks, compute_stream, copy_stream):
        _check(lib.hc_restore_context_static(self._h, store._h, seq_id, tok_begin, n_tok, pos_offset,
                                             _ptr(d_block_table), n_blocks, compute_stream,
                                             copy_stream))

    def restore_contexts(self, store, seq_ids, n_tok, d_block_tables, max_blocks, compute_stream,
                         copy_stream):
        import numpy as np
        ids = np.ascontiguousarray(seq_ids, dtype=np.int64)
        nt = np.ascontiguousarray(n_tok, dtype=np.int32)
        assert ids.shape == nt.shape
        _check(lib.hc_restore_contexts(self._h, store._h, len(ids), _ptr(ids), _ptr(nt),
                                       _ptr(d_block_tables), max_blocks, compute_stream, copy_stream))

    def restore_context_mixed(self, hidden_store, kv_store, l_h, seq_id, tok_begin, n_tok,
                              pos_offset, d_block_table, n_blocks, compute_stream, copy_stream):
        _check(lib.hc_restore_context_mixed(
            self._h, hidden_store._h if hidden_store is not None else None,
            kv_store._h if kv_store is not None else None, l_h, seq_id, tok_begin, n_tok,
            pos_offset, _ptr(d_block_table), n_blocks, compute_stream, copy_stream))

    def gather_kv(self, layer, d_rows, d_positions, n_tok, d_block_table, n_blocks, stream=0):
        _check(lib.hc_gather_kv(self._h, layer, _ptr(d_rows), _ptr(d_positions), n_tok,
                                _ptr(d_block_table), n_blocks, stream))

    def scatter_kv(self, layer, d_rows, d_positions, n_tok, d_block_table, n_blocks, stream=0):
        _check(lib.hc_scatter_kv(self._h, layer, _ptr(d_rows), _ptr(d_positions), n_tok,
                                 _ptr(d_block_table), n_blocks, stream))

    def set_loader(self, mode):
        _check(lib.hc_set_loader(self._h, mode))

    def set_split(self, mode):
        _check(lib.hc_set_split(self._h, mode))

    def timing_begin(self):
        _check(lib.hc_timing_begin(self._h))

    def timing_end_stats(self, stream=0):
        """(average, shortest, median) launch in ms and the launch count."""
        avg, mn, med, n = C.c_double(0), C.c_double(0), C.c_double(0), C.c_int32(0)
        _check(lib.hc_timing_end_stats(self._h, stream, C.byref(avg), C.byref(mn), C.byref(med), C.byref(n)))
        return avg.value, mn.value, med.value, n.value

    def timing_end(self, stream=0):
        avg, n = C.c_double(0), C.c_int32(0)
        _check(lib.hc_timing_end(self._h, stream, C.byref(avg), C.byref(n)))
        return avg.value, n.value


class Store:
    """Owner of an hc_store*."""

    def __init__(self, n_layers, d_model, chunk_tokens, capacity_chunks, pinned=True):
        h = C.c_void_p()
        _check(lib.hc_store_create_ex(n_layers, d_model, chunk_tokens, capacity_chunks,
                                      1 if pinned else 0, C.byref(h)))
        self._h = h
        self.n_layers, self.d_model, self.chunk_tokens = n_layers, d_model, chunk_tokens

    def destroy(self):
        if self._h:
            lib.hc_store_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def append(self, seq_id, layer, h_rows, n_tok):
        _check(lib.hc_store_append(self._h, seq_id, layer, _ptr(h_rows), n_tok))

    def tokens(self, seq_id, layer):
        return lib.hc_store_tokens(self._h, seq_id, layer)

    def chunk(self, seq_id, layer, chunk):
        """(host address, valid rows) of one chunk."""
        ptr, rows = C.c_void_p(), C.c_int32(0)
        _check(lib.hc_store_chunk(self._h, seq_id, layer, chunk, C.byref(ptr), C.byref(rows)))
        return ptr.value, rows.value

    def drop(self, seq_id):
        _check(lib.hc_store_drop(self._h, seq_id))


class Saver:
    """Owner of an hc_saver* (two-stage saving into a Store)."""

    def __init__(self, store, max_rows, n_slots=4, n_threads=8):
        h = C.c_void_p()
        _check(lib.hc_saver_create(store._h, max_rows, n_slots, n_threads, C.byref(h)))
        self._h = h
        self._store = store           # keep the store alive

    def destroy(self):
        if self._h:
            lib.hc_saver_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def save_layer(self, layer, d_hidden, n_rows, h_row_seq, compute_stream, down_stream):
        _check(lib.hc_saver_save_layer(self._h, layer, _ptr(d_hidden), n_rows, _ptr(h_row_seq),
                                       compute_stream, down_stream))

    def save_layer_deferred(self, layer, d_hidden, n_rows, h_row_seq, compute_stream, down_stream):
        _check(lib.hc_saver_save_layer_deferred(self._h, layer, _ptr(d_hidden), n_rows,
                                                _ptr(h_row_seq), compute_stream, down_stream))

    def fence(self, stream):
        _check(lib.hc_saver_fence(self._h, stream))

    def save_layer_host(self, layer, h_rows, n_rows, h_row_seq):
        _check(lib.hc_saver_save_layer_host(self._h, layer, _ptr(h_rows), n_rows, _ptr(h_row_seq)))

    def flush(self):
        _check(lib.hc_saver_flush(self._h))
