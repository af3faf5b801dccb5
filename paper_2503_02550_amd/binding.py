"""ctypes binding of libspecinf.so.  Argument marshalling only: every function forwards to the C entry point of
the same name (include/specinf.h); torch tensors are passed as their device addresses.  There is no fallback:
if the library is missing, importing this module raises."""
import ctypes as C
import os

# torch supplies the device memory and the streams this library works on, so both must use ONE HIP runtime: torch
# ships its own libamdhip64 and has to be loaded first, or the library would bind to a second runtime instance
# whose devices, streams and pointers are not torch's.
import torch  # noqa: F401  (load order)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecinf.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not built; run `python -m paper_2503_02550_amd.build`")
lib = C.CDLL(LIB_PATH)

u32, u64, i32, i64, f32, vp = C.c_uint32, C.c_uint64, C.c_int32, C.c_int64, C.c_float, C.c_void_p

# status codes / enums (mirrors of the header)
SIF_OK, SIF_W_SLO_RISK = 0, 1
SIF_E_INVAL, SIF_E_NOMEM, SIF_E_AGAIN, SIF_E_CANCELLED, SIF_E_TIMEOUT, SIF_E_DEVICE = -1, -2, -3, -4, -5, -6
SIF_F32, SIF_BF16 = 0, 1
SIF_STATUS_BUSY, SIF_STATUS_IDLE = 0, 1
SIF_A_ROW_K, SIF_A_ROW_M = 0, 1
SIF_B_ROW_K, SIF_B_ROW_N = 0, 1
SIF_EPI_NONE, SIF_EPI_BIAS, SIF_EPI_GELU, SIF_EPI_RESIDUAL, SIF_EPI_GELU_GRAD, SIF_EPI_OUT_F32, SIF_EPI_CAUSAL_SKIP = 0, 1, 2, 4, 8, 16, 32
SIF_MODEL_MLP, SIF_MODEL_DECODER, SIF_MODEL_ENCODER = 0, 1, 2
SIF_PAR_NONE, SIF_PAR_FIXED, SIF_PAR_DP, SIF_PAR_PP, SIF_PAR_TP = 0, 1, 2, 3, 4


class SifError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"sif status {status}: {text}")
        self.status = status


def last_error():
    return lib.sif_last_error().decode()


def check(status):
    if status < 0:
        raise SifError(status, last_error())
    return status


def ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def stream_ptr(s):
    if s is None:
        return None
    return s.cuda_stream if hasattr(s, "cuda_stream") else int(s)


class sif_alg1_params(C.Structure):
    _fields_ = [("alpha", u32), ("beta", u32), ("gamma_num", u32), ("gamma_den", u32), ("m", u32), ("reserved", u32),
                ("ll", u64), ("ul", u64), ("t0", u64)]


class sif_gemm_args(C.Structure):
    _fields_ = [("struct_size", u32), ("a_layout", u32), ("b_layout", u32), ("epilogue", u32),
                ("m", u32), ("n", u32), ("k", u32), ("lda", u32), ("ldb", u32), ("ldc", u32),
                ("batch_outer", u32), ("batch_inner", u32),
                ("a_stride_outer", i64), ("a_stride_inner", i64), ("b_stride_outer", i64), ("b_stride_inner", i64),
                ("c_stride_outer", i64), ("c_stride_inner", i64),
                ("alpha", f32), ("k_causal", u32),
                ("a_dev", vp), ("b_dev", vp), ("c_dev", vp), ("bias_dev", vp), ("res_dev", vp), ("aux_dev", vp),
                ("tile", u32), ("k_limit", u32)]


class sif_config(C.Structure):
    _fields_ = [("struct_size", u32), ("period_us", u32), ("window", u32), ("count_running", u32),
                ("alg1", sif_alg1_params), ("kernel_us_max", u32), ("collocate", u32), ("device_timed_bubbles", u32),
                ("allow_serial_streams", u32), ("device_capacity_bytes", u64),
                ("feedback", u32), ("feedback_eps_ppm", u32), ("feedback_add_ppm", u32), ("feedback_cap_ppm", u32),
                ("gate_spin_log2", u32), ("gate_spin_every", u32)]


class sif_model_shape(C.Structure):
    _fields_ = [("kind", u32), ("dtype", u32), ("n_layers", u32), ("d_model", u32), ("n_heads", u32), ("d_head", u32),
                ("d_ffn", u32), ("vocab", u32), ("max_pos", u32), ("d_in", u32), ("d_hidden", u32), ("d_out", u32),
                ("batch", u32), ("seq", u32)]


class sif_train_desc(C.Structure):
    _fields_ = [("struct_size", u32), ("par_mode", u32), ("shape", sif_model_shape), ("lr", f32),
                ("pp_stages", u32), ("pp_micro", u32), ("pp_stage", u32),
                ("bw_bytes_per_s", u64), ("fixed_bubble_ns", u64), ("pp_tf_ns", u64), ("pp_tb_ns", u64),
                ("master_dev", vp), ("workspace_dev", vp), ("workspace_bytes", u64), ("dp_bucket_bytes", u64)]


class sif_infer_desc(C.Structure):
    _fields_ = [("struct_size", u32), ("online", u32), ("shape", sif_model_shape), ("master_dev", vp),
                ("workspace_dev", vp), ("workspace_bytes", u64), ("peak_bytes", u64), ("coalesce", u32), ("reserved", u32)]


class sif_stats(C.Structure):
    _fields_ = [("struct_size", u32), ("status_now", u32), ("zc_now", u32), ("concurrent_share_ppm", u32), ("tokens_now", u64),
                ("steps", u64), ("step_ns_sum", u64), ("step_ns_last", u64), ("step_solo_ns", u64),
                ("bubble_ns", u64), ("filled_ns", u64), ("infer_busy_ns", u64),
                ("offline_samples", u64), ("offline_batches", u64),
                ("online_done", u64), ("online_p50_ns", u64), ("online_p95_ns", u64),
                ("kernels_launched", u64), ("kernels_skipped", u64), ("kernels_run", u64),
                ("gate_violations", u64), ("train_kernels", u64), ("periods", u64),
                ("gate_checked", u64), ("gate_unchecked", u64), ("gate_timeouts", u64)]


class sif_release_rec(C.Structure):
    _fields_ = [("period", u64), ("grant", u64), ("model", u32), ("charge", u32), ("launch", u32), ("kind", u32)]


class sif_trace_rec(C.Structure):
    _fields_ = [("kind", u32), ("id", u32), ("decision", u32), ("reserved", u32), ("t0_ns", u64), ("t1_ns", u64)]


def _sig(name, restype, *argtypes):
    f = getattr(lib, name)
    f.restype, f.argtypes = restype, list(argtypes)
    return f


P = C.POINTER
_sig("sif_last_error", C.c_char_p)
_sig("sif_abi_version", i32)
_sig("sif_zero_count", u32, P(u32), u32)
_sig("sif_alg1_step", i32, P(sif_alg1_params), u32, P(u64), P(u64), P(i32))
_sig("sif_kb_release", u32, P(u32), u32, u64, P(u64))
_sig("sif_online_pull_ok", i32, i32, u32, u64, u64)
_sig("sif_kb_charge", u32, u64, u64, u32)
_sig("sif_sched_run_trace", i32, P(sif_alg1_params), u32, P(u32), u32, P(u32), u32, P(u32), P(u64), P(u64), P(i32), P(u32))
_sig("sif_gate_violation", i32, u64, u64, u64)
_sig("sif_latency_bucket", u32, u64)
_sig("sif_latency_bucket_lower_ns", u64, u32)
_sig("sif_latency_buckets", u32)
_sig("sif_latency_percentile", u64, P(u64), u32, C.c_double)
_sig("sif_principle_1", i32, P(u64), u32, u64)
_sig("sif_principle_2", i32, u64, u64)
_sig("sif_collective_ns", u64, u64, u64)
_sig("sif_pp_1f1b_bubbles", i32, u32, u32, u32, u64, u64, P(i32), P(i32), P(u64), u32)
_sig("sif_feedback_share", u32, u32, u64, u64, u32, u32, u32)
_sig("sif_concurrent_account", u64, u64, u32, u64, u64)
_sig("sif_dp_gradient_buckets", i32, P(u64), u32, u64, P(u32))
_sig("sif_dp_overlapped_wait", u64, P(u64), P(u64), u32, u64)
_sig("sif_k_gemm_bf16", i32, P(sif_gemm_args), vp)
_sig("sif_k_gemm_f32", i32, vp, i64, i64, vp, i64, i64, vp, i64, u32, u32, u32, u32, vp, vp, vp)
_sig("sif_k_layernorm_fwd", i32, vp, vp, vp, vp, vp, vp, u32, u32, vp)
_sig("sif_k_layernorm_bwd", i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u32, u32, vp)
_sig("sif_colsum_parts", u32, u32)
_sig("sif_k_colsum", i32, vp, u32, vp, vp, u32, u32, vp)
_sig("sif_k_colsum_static", i32, vp, u32, vp, u32, u32, vp)
_sig("sif_colsum_static_max_floats", u64)
_sig("sif_k_softmax_fwd", i32, vp, vp, u32, u32, u32, u32, u32, u32, vp)
_sig("sif_k_softmax_bwd", i32, vp, vp, vp, u32, u32, u32, u32, f32, u32, vp)
_sig("sif_k_embed_fwd", i32, vp, vp, vp, vp, u32, u32, u32, u32, vp)
_sig("sif_k_embed_bwd", i32, vp, vp, vp, vp, u32, u32, u32, u32, vp)
_sig("sif_k_xent_fwd_bwd", i32, vp, vp, vp, u32, u32, u32, vp)
_sig("sif_k_reduce_sum", i32, vp, vp, u32, f32, vp)
_sig("sif_k_sgd_bf16", i32, vp, vp, vp, u64, f32, vp)
_sig("sif_k_sgd_f32", i32, vp, vp, u64, f32, vp)
_sig("sif_k_mse_fwd_bwd", i32, vp, vp, vp, vp, u32, vp)
_sig("sif_k_colsum_f32", i32, vp, u32, vp, u32, u32, vp)


# ---- pure host rules ------------------------------------------------------------------------------------
def sif_zero_count(counts):
    arr = (u32 * len(counts))(*counts)
    return lib.sif_zero_count(arr, len(counts))


def sif_alg1_step(params, zc, pool):
    """Returns (pool', grant, status)."""
    p, g, s = u64(pool), u64(0), i32(0)
    check(lib.sif_alg1_step(C.byref(params), zc, C.byref(p), C.byref(g), C.byref(s)))
    return p.value, g.value, s.value


def sif_kb_release(costs, balance):
    arr = (u32 * max(1, len(costs)))(*costs)
    left = u64(0)
    n = lib.sif_kb_release(arr, len(costs), balance, C.byref(left))
    return n, left.value


def sif_kb_charge(predicted_us, ul, m):
    return lib.sif_kb_charge(predicted_us, ul, m)


def sif_sched_run_trace(params, window, counts, costs):
    """Monitor -> Algorithm 1 -> offline barrier over a trace of per-period counts.  Returns one tuple per period:
    (Z_c, pool, grant, status, kernels forwarded)."""
    n, nc = len(counts), len(costs)
    cnt, cst = (u32 * max(1, n))(*counts), (u32 * max(1, nc))(*costs)
    zc, pool, grant, status, rel = (u32 * max(1, n))(), (u64 * max(1, n))(), (u64 * max(1, n))(), (i32 * max(1, n))(), (u32 * max(1, n))()
    check(lib.sif_sched_run_trace(C.byref(params), window, cnt, n, cst, nc, zc, pool, grant, status, rel))
    return [(zc[i], pool[i], grant[i], status[i], rel[i]) for i in range(n)]


def sif_gate_violation(t0, bubble_begin, bubble_end):
    return bool(lib.sif_gate_violation(t0, bubble_begin, bubble_end))


def sif_latency_bucket(ns):
    return lib.sif_latency_bucket(ns)


def sif_latency_bucket_lower_ns(bucket):
    return lib.sif_latency_bucket_lower_ns(bucket)


def sif_latency_buckets():
    return lib.sif_latency_buckets()


def sif_latency_percentile(counts, p):
    arr = (u64 * max(1, len(counts)))(*counts)
    return lib.sif_latency_percentile(arr, len(counts), p)


def sif_online_pull_ok(status, queue_len, remaining_ns, request_ns):
    return bool(lib.sif_online_pull_ok(status, queue_len, remaining_ns, request_ns))


def sif_principle_1(peaks, capacity):
    arr = (u64 * max(1, len(peaks)))(*peaks)
    return bool(lib.sif_principle_1(arr, len(peaks), capacity))


def sif_principle_2(min_exec_ns, max_bubble_ns):
    return bool(lib.sif_principle_2(min_exec_ns, max_bubble_ns))


def sif_collective_ns(n_bytes, bw):
    return lib.sif_collective_ns(n_bytes, bw)


def sif_pp_1f1b_bubbles(stage, n_stages, n_micro, tf_ns, tb_ns, cap=64):
    kind, idx, ns = (i32 * cap)(), (i32 * cap)(), (u64 * cap)()
    n = check(lib.sif_pp_1f1b_bubbles(stage, n_stages, n_micro, tf_ns, tb_ns, kind, idx, ns, cap))
    return [(kind[i], idx[i], ns[i]) for i in range(min(n, cap))]


def sif_feedback_share(share_ppm, step_ns, ref_ns, eps_ppm, add_ppm, cap_ppm=1_000_000):
    return lib.sif_feedback_share(share_ppm, step_ns, ref_ns, eps_ppm, add_ppm, cap_ppm)


def sif_concurrent_account(balance_ns, share_ppm, period_ns, burst_ns):
    return lib.sif_concurrent_account(balance_ns, share_ppm, period_ns, burst_ns)


def sif_dp_gradient_buckets(group_bytes, cap_bytes):
    """Bucket number of every group."""
    n = len(group_bytes)
    gb, out = (u64 * max(n, 1))(*group_bytes), (u32 * max(n, 1))()
    nb = check(lib.sif_dp_gradient_buckets(gb, n, cap_bytes, out))
    return nb, [out[i] for i in range(n)]


def sif_dp_overlapped_wait(ready_ns, dur_ns, end_ns):
    n = len(ready_ns)
    assert len(dur_ns) == n
    return lib.sif_dp_overlapped_wait((u64 * max(n, 1))(*ready_ns), (u64 * max(n, 1))(*dur_ns), n, end_ns)


# ---- single kernels -------------------------------------------------------------------------------------
def gemm_args(a, b, c, m, n, k, lda, ldb, ldc, a_layout=SIF_A_ROW_K, b_layout=SIF_B_ROW_K, epilogue=0,
              bias=None, res=None, aux=None, alpha=1.0, batch_outer=1, batch_inner=1,
              a_strides=(0, 0), b_strides=(0, 0), c_strides=(0, 0), k_causal=0, tile=0, k_limit=0):
    """A filled sif_gemm_args (argument marshalling only)."""
    g = sif_gemm_args()
    g.struct_size = C.sizeof(sif_gemm_args)
    g.a_layout, g.b_layout, g.epilogue = a_layout, b_layout, epilogue
    g.m, g.n, g.k, g.lda, g.ldb, g.ldc = m, n, k, lda, ldb, ldc
    g.batch_outer, g.batch_inner = batch_outer, batch_inner
    g.a_stride_outer, g.a_stride_inner = a_strides
    g.b_stride_outer, g.b_stride_inner = b_strides
    g.c_stride_outer, g.c_stride_inner = c_strides
    g.alpha, g.k_causal, g.tile, g.k_limit = alpha, k_causal, tile, k_limit
    g.a_dev, g.b_dev, g.c_dev, g.bias_dev, g.res_dev, g.aux_dev = ptr(a), ptr(b), ptr(c), ptr(bias), ptr(res), ptr(aux)
    return g


def sif_k_gemm_bf16(*args, stream=None, **kw):
    g = gemm_args(*args, **kw)
    return check(lib.sif_k_gemm_bf16(C.byref(g), stream_ptr(stream)))


_sig("sif_k_gemm_bf16_group_bytes", u64, u32)
_sig("sif_k_gemm_bf16_group", i32, P(sif_gemm_args), u32, vp, vp)


def sif_k_gemm_bf16_group_bytes(n):
    return lib.sif_k_gemm_bf16_group_bytes(n)


def sif_k_gemm_bf16_group(products, records, stream=None):
    """products: sif_gemm_args from gemm_args(); records: device memory of sif_k_gemm_bf16_group_bytes(len(products)) bytes."""
    arr = (sif_gemm_args * max(1, len(products)))(*products)
    return check(lib.sif_k_gemm_bf16_group(arr, len(products), ptr(records), stream_ptr(stream)))


def sif_k_gemm_f32(a, a_sm, a_sk, b, b_sk, b_sn, c, ldc, m, n, k, epilogue=0, bias=None, aux=None, stream=None):
    return check(lib.sif_k_gemm_f32(ptr(a), a_sm, a_sk, ptr(b), b_sk, b_sn, ptr(c), ldc, m, n, k, epilogue, ptr(bias),
                                    ptr(aux), stream_ptr(stream)))


def sif_k_layernorm_fwd(x, g, b, y, mean, rstd, rows, d, stream=None):
    return check(lib.sif_k_layernorm_fwd(ptr(x), ptr(g), ptr(b), ptr(y), ptr(mean), ptr(rstd), rows, d, stream_ptr(stream)))


def sif_k_layernorm_bwd(dy, x, g, mean, rstd, res, dx, dg, db, part, rows, d, dsum=None, stream=None):
    return check(lib.sif_k_layernorm_bwd(ptr(dy), ptr(x), ptr(g), ptr(mean), ptr(rstd), ptr(res), ptr(dx), ptr(dg),
                                         ptr(db), ptr(dsum) if dsum is not None else None, ptr(part), rows, d, stream_ptr(stream)))


def sif_colsum_parts(rows):
    return lib.sif_colsum_parts(rows)


def sif_k_colsum(x, ld, out, part, rows, n, stream=None):
    return check(lib.sif_k_colsum(ptr(x), ld, ptr(out), ptr(part), rows, n, stream_ptr(stream)))


def sif_k_colsum_static(x, ld, out, rows, n, stream=None):
    return check(lib.sif_k_colsum_static(ptr(x), ld, ptr(out), rows, n, stream_ptr(stream)))


def sif_colsum_static_max_floats():
    return lib.sif_colsum_static_max_floats()


def sif_k_softmax_fwd(s, p, batch, rows, cols, ld_s, ld_p, causal, stream=None):
    return check(lib.sif_k_softmax_fwd(ptr(s), ptr(p), batch, rows, cols, ld_s, ld_p, causal, stream_ptr(stream)))


def sif_k_softmax_bwd(dp, p, ds, batch, rows, cols, ld, scale, causal, stream=None):
    return check(lib.sif_k_softmax_bwd(ptr(dp), ptr(p), ptr(ds), batch, rows, cols, ld, scale, causal, stream_ptr(stream)))


def sif_k_embed_fwd(ids, wte, wpe, x, vocab, tokens, seq, d, stream=None):
    return check(lib.sif_k_embed_fwd(ptr(ids), ptr(wte), ptr(wpe), ptr(x), vocab, tokens, seq, d, stream_ptr(stream)))


def sif_k_embed_bwd(ids, dx, dwte, dwpe, vocab, tokens, seq, d, stream=None):
    return check(lib.sif_k_embed_bwd(ptr(ids), ptr(dx), ptr(dwte), ptr(dwpe), vocab, tokens, seq, d, stream_ptr(stream)))


def sif_k_xent_fwd_bwd(logits, targets, loss, tokens, vocab, ld, stream=None):
    return check(lib.sif_k_xent_fwd_bwd(ptr(logits), ptr(targets), ptr(loss), tokens, vocab, ld, stream_ptr(stream)))


def sif_k_reduce_sum(x, out, n, scale, stream=None):
    return check(lib.sif_k_reduce_sum(ptr(x), ptr(out), n, scale, stream_ptr(stream)))


def sif_k_sgd_bf16(master, grad, work, n, lr, stream=None):
    return check(lib.sif_k_sgd_bf16(ptr(master), ptr(grad), ptr(work), n, lr, stream_ptr(stream)))


def sif_k_sgd_f32(p, g, n, lr, stream=None):
    return check(lib.sif_k_sgd_f32(ptr(p), ptr(g), n, lr, stream_ptr(stream)))


def sif_k_mse_fwd_bwd(y, t, d, loss, n, stream=None):
    return check(lib.sif_k_mse_fwd_bwd(ptr(y), ptr(t), ptr(d), ptr(loss), n, stream_ptr(stream)))


def sif_k_colsum_f32(x, ld, out, rows, n, stream=None):
    return check(lib.sif_k_colsum_f32(ptr(x), ld, ptr(out), rows, n, stream_ptr(stream)))


# ---- runtime ----------------------------------------------------------------------------------------------
_sig("sif_now_ns", u64)
_sig("sif_default_config", i32, P(sif_config))
_sig("sif_ctx_workspace_bytes", u64)
_sig("sif_create", i32, P(sif_config), vp, vp, vp, u64, P(vp))
_sig("sif_destroy", i32, vp)
_sig("sif_set_collocate", i32, vp, u32)
_sig("sif_model_n_params", u64, P(sif_model_shape))
_sig("sif_train_workspace_bytes", u64, P(sif_train_desc))
_sig("sif_register_training_step", i32, vp, P(sif_train_desc), P(i32))
_sig("sif_run_training_step", i32, vp, i32, vp, vp, vp)
_sig("sif_sync_training", i32, vp)
_sig("sif_train_tensor", i32, vp, i32, C.c_char_p, i32, P(vp), P(u64))
_sig("sif_infer_workspace_bytes", u64, P(sif_infer_desc))
_sig("sif_register_inference_model", i32, vp, P(sif_infer_desc), P(i32))
_sig("sif_calibrate", i32, vp, u32, vp, vp)
_sig("sif_submit_offline_batch", i32, vp, i32, vp, vp, u32, u32, P(u64))
_sig("sif_submit_online_request", i32, vp, i32, vp, vp, u32, u64, P(u64))
_sig("sif_wait", i32, vp, u64, u64)
_sig("sif_poll_stats", i32, vp, P(sif_stats))
_sig("sif_reset_stats", i32, vp)
_sig("sif_read_trace", i32, vp, u32, P(sif_trace_rec), u32, P(u32))
_sig("sif_read_release_log", i32, vp, P(sif_release_rec), u32, P(u32))
_sig("sif_read_latency_histogram", i32, vp, P(u64), u32, P(u32))


def sif_now_ns():
    return lib.sif_now_ns()


def sif_default_config():
    cfg = sif_config()
    check(lib.sif_default_config(C.byref(cfg)))
    return cfg


def sif_ctx_workspace_bytes():
    return lib.sif_ctx_workspace_bytes()


def sif_create(cfg, train_stream, infer_stream, workspace, workspace_bytes):
    out = vp()
    check(lib.sif_create(C.byref(cfg), stream_ptr(train_stream), stream_ptr(infer_stream), ptr(workspace), workspace_bytes,
                         C.byref(out)))
    return out


def sif_destroy(ctx):
    return check(lib.sif_destroy(ctx))


def sif_set_collocate(ctx, on):
    return check(lib.sif_set_collocate(ctx, 1 if on else 0))


def sif_model_n_params(shape):
    return lib.sif_model_n_params(C.byref(shape))


def sif_train_workspace_bytes(desc):
    n = lib.sif_train_workspace_bytes(C.byref(desc))
    if n == 0:
        raise SifError(SIF_E_INVAL, last_error())
    return n


def sif_register_training_step(ctx, desc):
    h = i32(-1)
    check(lib.sif_register_training_step(ctx, C.byref(desc), C.byref(h)))
    return h.value


def sif_run_training_step(ctx, h, inputs, targets, loss=None):
    return check(lib.sif_run_training_step(ctx, h, ptr(inputs), ptr(targets), ptr(loss)))


def sif_sync_training(ctx):
    return check(lib.sif_sync_training(ctx))


def sif_train_tensor(ctx, h, name, layer=0):
    """Returns (device address, element count)."""
    p, n = vp(), u64(0)
    check(lib.sif_train_tensor(ctx, h, name.encode(), layer, C.byref(p), C.byref(n)))
    return p.value, n.value


def sif_infer_workspace_bytes(desc):
    return lib.sif_infer_workspace_bytes(C.byref(desc))


def sif_register_inference_model(ctx, desc):
    h = i32(-1)
    check(lib.sif_register_inference_model(ctx, C.byref(desc), C.byref(h)))
    return h.value


def sif_calibrate(ctx, iters, train_inputs=None, train_targets=None):
    return check(lib.sif_calibrate(ctx, iters, ptr(train_inputs), ptr(train_targets)))


def sif_submit_offline_batch(ctx, model, inp, out, batch, seq):
    t = u64(0)
    check(lib.sif_submit_offline_batch(ctx, model, ptr(inp), ptr(out), batch, seq, C.byref(t)))
    return t.value


def sif_submit_online_request(ctx, model, inp, out, seq, t_arrival_ns=0):
    t = u64(0)
    check(lib.sif_submit_online_request(ctx, model, ptr(inp), ptr(out), seq, t_arrival_ns, C.byref(t)))
    return t.value


def sif_wait(ctx, ticket, timeout_ns=10_000_000_000):
    return check(lib.sif_wait(ctx, ticket, timeout_ns))


def sif_poll_stats(ctx):
    s = sif_stats()
    s.struct_size = C.sizeof(sif_stats)
    check(lib.sif_poll_stats(ctx, C.byref(s)))
    return s


def sif_reset_stats(ctx):
    return check(lib.sif_reset_stats(ctx))


def sif_read_trace(ctx, which, cap=65535):
    """Returns a list of (kind, id, decision, launch number, t0_ns, t1_ns), oldest first."""
    arr = (sif_trace_rec * cap)()
    n = u32(0)
    check(lib.sif_read_trace(ctx, which, arr, cap, C.byref(n)))
    return [(arr[i].kind, arr[i].id, arr[i].decision, arr[i].reserved, arr[i].t0_ns, arr[i].t1_ns) for i in range(n.value)]


def sif_read_release_log(ctx, cap=65536):
    """Returns a list of (period, grant, model, charge, launch number, kind), oldest first."""
    arr = (sif_release_rec * cap)()
    n = u32(0)
    check(lib.sif_read_release_log(ctx, arr, cap, C.byref(n)))
    return [(arr[i].period, arr[i].grant, arr[i].model, arr[i].charge, arr[i].launch, arr[i].kind) for i in range(n.value)]


def sif_read_latency_histogram(ctx):
    """Counts per bucket of the online latency histogram."""
    cap = lib.sif_latency_buckets()
    arr = (u64 * cap)()
    n = u32(0)
    check(lib.sif_read_latency_histogram(ctx, arr, cap, C.byref(n)))
    return [arr[i] for i in range(n.value)]


_sig("sif_profile_gemm", i32, vp, u32)
_sig("sif_profile_read", i32, vp, P(u64), P(C.c_double), P(C.c_double))


def sif_profile_gemm(ctx, on):
    return check(lib.sif_profile_gemm(ctx, int(on)))


def sif_profile_read(ctx):
    """Per GEMM layout variant (a_layout*2 + b_layout): (launches, algorithmic flops, seconds)."""
    n, f, s = (u64 * 4)(), (C.c_double * 4)(), (C.c_double * 4)()
    check(lib.sif_profile_read(ctx, n, f, s))
    return [(n[i], f[i], s[i]) for i in range(4)]


def sif_abi_version():
    return lib.sif_abi_version()


_sig("sif_train_op_name", C.c_char_p, vp, i32, u32)
_sig("sif_train_dp_bucket", i32, vp, i32, u32, P(u64), P(u32))


def sif_train_dp_buckets(ctx, h):
    """[(bytes, index of the launch that finalizes the bucket)] of a step with a bucketed gradient exchange."""
    out = []
    while True:
        b, r = u64(), u32()
        if lib.sif_train_dp_bucket(ctx, h, len(out), C.byref(b), C.byref(r)) != 0:
            return out
        out.append((b.value, r.value))


def sif_train_op_name(ctx, h, index):
    n = lib.sif_train_op_name(ctx, h, index)
    return n.decode() if n else None


_sig("sif_k_attn_fwd", i32, vp, vp, vp, u32, u32, u32, u32, u32, u32, u32, vp)
_sig("sif_k_attn_bwd", i32, vp, vp, vp, vp, vp, vp, u32, u32, u32, u32, u32, u32, u32, u32, vp)


def sif_k_attn_fwd(qkv, o, batch, seq, heads, d_head, ld_qkv, ld_o, causal, lse=None, stream=None):
    return check(lib.sif_k_attn_fwd(ptr(qkv), ptr(o), ptr(lse) if lse is not None else None, batch, seq, heads, d_head, ld_qkv, ld_o,
                                    causal, stream_ptr(stream)))


_sig("sif_k_attn_fwd_varlen", i32, vp, vp, P(u32), u32, u32, u32, u32, u32, u32, vp)


def sif_k_attn_fwd_varlen(qkv, o, seq_starts, heads, d_head, ld_qkv, ld_o, causal, stream=None):
    n = len(seq_starts) - 1
    arr = (u32 * (n + 1))(*seq_starts)
    return check(lib.sif_k_attn_fwd_varlen(ptr(qkv), ptr(o), arr, n, heads, d_head, ld_qkv, ld_o, causal, stream_ptr(stream)))


def sif_k_attn_bwd(qkv, o, d_o, lse, delta, dqkv, batch, seq, heads, d_head, ld_qkv, ld_o, ld_dqkv, causal, stream=None):
    return check(lib.sif_k_attn_bwd(ptr(qkv), ptr(o), ptr(d_o), ptr(lse), ptr(delta), ptr(dqkv), batch, seq, heads, d_head, ld_qkv, ld_o,
                                    ld_dqkv, causal, stream_ptr(stream)))
