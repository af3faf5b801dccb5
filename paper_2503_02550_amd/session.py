"""Plumbing around the C ABI for Python callers: torch supplies the device memory and the two streams, every
computation happens inside libspecinf.so.  Used by the tests, the smoke check and the benchmark."""
import ctypes as C

import numpy as np
import torch

from . import binding as B
from . import params as P


def _u8(nbytes, dev):
    return torch.zeros(int(nbytes) + 256, dtype=torch.uint8, device=dev)


def _aligned(t):
    """256-byte aligned address inside a uint8 tensor that was over-allocated by 256 bytes."""
    return (t.data_ptr() + 255) & ~255


class Session:
    def __init__(self, cfg=None, device="cuda:0"):
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.cfg = cfg if cfg is not None else B.sif_default_config()
        self._ws = _u8(B.sif_ctx_workspace_bytes(), self.dev)
        self.st_train = torch.cuda.Stream(device=self.dev)
        self.ctx = None
        for _ in range(16):      # sif_create refuses a stream pair that shares a hardware queue (SIF_E_AGAIN)
            self.st_infer = torch.cuda.Stream(device=self.dev)
            torch.cuda.synchronize()
            try:
                self.ctx = B.sif_create(self.cfg, self.st_train, self.st_infer, _aligned(self._ws), B.sif_ctx_workspace_bytes())
                break
            except B.SifError as e:
                if e.status != B.SIF_E_AGAIN:
                    raise
        if self.ctx is None:
            raise RuntimeError("no pair of concurrent streams found")
        self.train = None
        self.models = []

    # ---- training --------------------------------------------------------------------------------------
    def register_training(self, shape, master_flat, par_mode=B.SIF_PAR_NONE, lr=0.01, bw_bytes_per_s=0, fixed_bubble_ns=0,
                          pp_stages=0, pp_micro=0, pp_stage=0, pp_tf_ns=0, pp_tb_ns=0, dp_bucket_bytes=0):
        d = B.sif_train_desc()
        d.struct_size = C.sizeof(d)
        d.par_mode, d.shape, d.lr = par_mode, shape, lr
        d.bw_bytes_per_s, d.fixed_bubble_ns = bw_bytes_per_s, fixed_bubble_ns
        d.pp_stages, d.pp_micro, d.pp_stage, d.pp_tf_ns, d.pp_tb_ns = pp_stages, pp_micro, pp_stage, pp_tf_ns, pp_tb_ns
        d.dp_bucket_bytes = dp_bucket_bytes
        need = B.sif_train_workspace_bytes(d)
        master = torch.from_numpy(np.ascontiguousarray(master_flat, dtype=np.float32)).to(self.dev)
        ws = _u8(need, self.dev)
        torch.cuda.synchronize()
        d.master_dev, d.workspace_dev, d.workspace_bytes = master.data_ptr(), _aligned(ws), need
        h = B.sif_register_training_step(self.ctx, d)
        self.train = dict(handle=h, shape=shape, master=master, ws=ws, desc=d)
        return h

    def step(self, inputs, targets, loss=None):
        return B.sif_run_training_step(self.ctx, self.train["handle"], inputs, targets, loss)

    def sync(self):
        B.sif_sync_training(self.ctx)
        torch.cuda.synchronize()

    def train_tensor(self, name, layer=0, dtype=torch.bfloat16):
        """A torch view (no copy) of a named tensor inside the training workspace or the master array."""
        addr, n = B.sif_train_tensor(self.ctx, self.train["handle"], name, layer)
        for base in (self.train["ws"], self.train["master"]):
            b0 = base.data_ptr()
            if b0 <= addr < b0 + base.numel() * base.element_size():
                raw = base.view(torch.uint8).reshape(-1)
                off = addr - b0
                return raw[off:off + n * torch.empty((), dtype=dtype).element_size()].view(dtype)
        raise RuntimeError("tensor outside the known buffers")

    # ---- inference -------------------------------------------------------------------------------------
    def register_inference(self, shape, master_flat, online=False, peak_bytes=None, coalesce=0):
        d = B.sif_infer_desc()
        d.struct_size = C.sizeof(d)
        d.online, d.shape, d.coalesce = (1 if online else 0), shape, coalesce
        need = B.sif_infer_workspace_bytes(d)
        master = torch.from_numpy(np.ascontiguousarray(master_flat, dtype=np.float32)).to(self.dev)
        ws = _u8(need, self.dev)
        torch.cuda.synchronize()
        d.master_dev, d.workspace_dev, d.workspace_bytes = master.data_ptr(), _aligned(ws), need
        d.peak_bytes = peak_bytes if peak_bytes is not None else need + master.numel() * 4
        h = B.sif_register_inference_model(self.ctx, d)
        self.models.append(dict(handle=h, shape=shape, master=master, ws=ws, desc=d))
        return h

    def submit_offline(self, model, inp, out, batch, seq=1):
        return B.sif_submit_offline_batch(self.ctx, model, inp, out, batch, seq)

    def submit_online(self, model, inp, out, seq, t_arrival_ns=0):
        return B.sif_submit_online_request(self.ctx, model, inp, out, seq, t_arrival_ns)

    def wait(self, ticket, timeout_s=10.0):
        return B.sif_wait(self.ctx, ticket, int(timeout_s * 1e9))

    def stats(self):
        return B.sif_poll_stats(self.ctx)

    def close(self):
        if self.ctx is not None:
            B.sif_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()


def decoder_shape(cfg):
    return P.make_shape(B.SIF_MODEL_DECODER, B.SIF_BF16, n_layers=cfg["n_layers"], d_model=cfg["d_model"], n_heads=cfg["n_heads"],
                        d_head=cfg["d_head"], d_ffn=cfg["d_ffn"], vocab=cfg.get("vocab", 0), max_pos=cfg.get("max_pos", 0),
                        batch=cfg["batch"], seq=cfg["seq"])


def encoder_shape(cfg):
    return P.make_shape(B.SIF_MODEL_ENCODER, B.SIF_BF16, n_layers=cfg["n_layers"], d_model=cfg["d_model"], n_heads=cfg["n_heads"],
                        d_head=cfg["d_head"], d_ffn=cfg["d_ffn"], vocab=cfg["vocab"], max_pos=cfg["max_pos"],
                        batch=cfg["batch"], seq=cfg["seq"])


def mlp_shape(d_in, d_hidden, d_out, batch):
    return P.make_shape(B.SIF_MODEL_MLP, B.SIF_F32, d_in=d_in, d_hidden=d_hidden, d_out=d_out, batch=batch)
