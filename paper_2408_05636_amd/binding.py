"""ctypes binding of libspecdiff.so: argument marshalling only.

PyTorch appears here only as the owner of device memory (weights, workspace, test rows) and of
the HIP stream; every step of the round runs inside the library's kernels.  There is no CPU
fallback: loading fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Sequence, Tuple

import numpy as np

from .synth import ModelConfig, weight_specs

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecdiff.so")

SD_OK = 0
STATUS_NAMES = {0: "SD_OK", 1: "SD_ERR_ARG", 2: "SD_ERR_SHAPE", 3: "SD_ERR_TOKEN", 4: "SD_ERR_STATE",
                5: "SD_ERR_WORKSPACE", 6: "SD_ERR_HIP"}
EXPORTS = ["sd_vocab_pad", "sd_weight_count", "sd_weight_desc", "sd_weight_bytes", "sd_workspace_bytes", "sd_create",
           "sd_destroy", "sd_last_error", "sd_prefill", "sd_draft", "sd_verify", "sd_round", "sd_drafter_logits",
           "sd_target_logits", "sd_sampling_scratch_bytes", "sd_unmask_sample", "sd_accept_resample", "sd_linear",
           "sd_profile_begin", "sd_profile_end", "sd_profile_count", "sd_profile_entry", "sd_set_graph_replay", "sd_set_linear_variant", "sd_norm_linear",
           "sd_set_linear_split", "sd_linear_split_ticket_bytes", "sd_commit", "sd_set_greedy", "sd_set_step_skipping", "sd_steps_run", "sd_norm_linear_scratch_floats", "sd_linear_resid_norm",
           "sd_graph_stats", "sd_graph_error", "sd_sps_workspace_bytes", "sd_sps_attach", "sd_sps_draft", "sd_sps_round", "sd_sps_logits", "sd_static_scratch_bytes", "sd_accept_resample_static"]


class SdModelConfig(C.Structure):
    _fields_ = [("arch", C.c_int32), ("dtype", C.c_int32), ("n_layer", C.c_int32), ("d_model", C.c_int32),
                ("n_head", C.c_int32), ("n_kv_head", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("n_ctx", C.c_int32), ("bidirectional", C.c_int32), ("norm_eps", C.c_float), ("rope_theta", C.c_float)]


class SdError(RuntimeError):
    def __init__(self, code: int, where: str, msg: str = ""):
        self.code = code
        super().__init__(f"{where}: {STATUS_NAMES.get(code, code)} {msg}")


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_05636_amd.build` "
                               "(there is no fallback path)")
        # torch ships its own HIP runtime (same soname): load it first so that the library binds to
        # the runtime that owns torch's device memory and streams, whatever the import order.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        i32, i64, u64, vp, ip, fp = C.c_int32, C.c_int64, C.c_uint64, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float)
        cfgp = C.POINTER(SdModelConfig)
        L.sd_vocab_pad.restype = i32; L.sd_vocab_pad.argtypes = [i32]
        L.sd_weight_count.restype = i32; L.sd_weight_count.argtypes = [cfgp]
        L.sd_weight_desc.restype = i32
        L.sd_weight_desc.argtypes = [cfgp, i32, C.c_char_p, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i64)]
        L.sd_weight_bytes.restype = i64; L.sd_weight_bytes.argtypes = [cfgp]
        L.sd_workspace_bytes.restype = i64; L.sd_workspace_bytes.argtypes = [cfgp, cfgp, i32, i32]
        L.sd_create.restype = i32
        L.sd_create.argtypes = [cfgp, cfgp, vp, vp, i32, i32, vp, i64, vp, C.POINTER(vp)]
        L.sd_destroy.restype = None; L.sd_destroy.argtypes = [vp]
        L.sd_last_error.restype = C.c_char_p; L.sd_last_error.argtypes = [vp]
        L.sd_prefill.restype = i32; L.sd_prefill.argtypes = [vp, i32, ip, ip]
        L.sd_draft.restype = i32; L.sd_draft.argtypes = [vp, i32, ip, ip, i32, i32, u64, ip, fp, C.POINTER(vp)]
        L.sd_verify.restype = i32; L.sd_verify.argtypes = [vp, i32, ip, ip, i32, ip, vp, u64, ip, ip]
        L.sd_round.restype = i32; L.sd_round.argtypes = [vp, i32, ip, ip, i32, i32, u64, ip, ip, ip]
        L.sd_drafter_logits.restype = i32; L.sd_drafter_logits.argtypes = [vp, i32, ip, ip, i32, i32, i32, C.POINTER(vp)]
        L.sd_target_logits.restype = i32; L.sd_target_logits.argtypes = [vp, i32, ip, ip, i32, ip, C.POINTER(vp)]
        L.sd_sampling_scratch_bytes.restype = i64; L.sd_sampling_scratch_bytes.argtypes = [i32, i32]
        L.sd_unmask_sample.restype = i32
        L.sd_unmask_sample.argtypes = [vp, i32, i32, i32, i32, u64, vp, vp, vp, vp, i64, vp]
        L.sd_accept_resample.restype = i32
        L.sd_accept_resample.argtypes = [vp, vp, vp, i32, i32, i32, u64, vp, vp, vp, i64, vp]
        L.sd_static_scratch_bytes.restype = i64; L.sd_static_scratch_bytes.argtypes = []
        L.sd_accept_resample_static.restype = i32
        L.sd_accept_resample_static.argtypes = [vp, vp, vp, i32, i32, i32, u64, vp, vp, vp]
        L.sd_linear.restype = i32
        L.sd_linear.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, i64, vp]
        L.sd_set_linear_split.restype = i32; L.sd_set_linear_split.argtypes = [i32]
        L.sd_norm_linear_scratch_floats.restype = i64; L.sd_norm_linear_scratch_floats.argtypes = [i32, i32, i32]
        L.sd_linear_resid_norm.restype = i32
        L.sd_linear_resid_norm.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, i64, vp]
        L.sd_commit.restype = i32; L.sd_commit.argtypes = [vp, i32, C.POINTER(C.c_int32)]
        L.sd_set_greedy.restype = i32; L.sd_set_greedy.argtypes = [vp, i32]
        L.sd_set_step_skipping.restype = i32; L.sd_set_step_skipping.argtypes = [vp, i32]
        L.sd_steps_run.restype = i32; L.sd_steps_run.argtypes = [vp]
        L.sd_linear_split_ticket_bytes.restype = i64; L.sd_linear_split_ticket_bytes.argtypes = []
        L.sd_set_graph_replay.restype = i32; L.sd_set_graph_replay.argtypes = [vp, i32]
        L.sd_set_linear_variant.restype = i32; L.sd_set_linear_variant.argtypes = [i32]
        L.sd_sps_workspace_bytes.restype = i64; L.sd_sps_workspace_bytes.argtypes = [vp, cfgp]
        L.sd_sps_attach.restype = i32; L.sd_sps_attach.argtypes = [vp, cfgp, vp, vp, i64]
        L.sd_sps_draft.restype = i32; L.sd_sps_draft.argtypes = [vp, i32, ip, ip, i32, u64, ip, fp, C.POINTER(vp)]
        L.sd_sps_round.restype = i32; L.sd_sps_round.argtypes = [vp, i32, ip, ip, i32, u64, ip, ip, ip]
        L.sd_sps_logits.restype = i32; L.sd_sps_logits.argtypes = [vp, i32, ip, ip, C.POINTER(vp)]
        L.sd_graph_stats.restype = i32
        L.sd_graph_stats.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
        L.sd_graph_error.restype = C.c_char_p; L.sd_graph_error.argtypes = [vp]
        L.sd_norm_linear.restype = i32
        L.sd_norm_linear.argtypes = [i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, C.c_float, vp, vp, i64, vp]
        L.sd_profile_begin.restype = i32; L.sd_profile_begin.argtypes = [vp]
        L.sd_profile_end.restype = i32; L.sd_profile_end.argtypes = [vp]
        L.sd_profile_count.restype = i32; L.sd_profile_count.argtypes = [vp]
        L.sd_profile_entry.restype = i32
        L.sd_profile_entry.argtypes = [vp, i32, C.c_char_p, i32, C.POINTER(i64), C.POINTER(C.c_double),
                                       C.POINTER(C.c_double), C.POINTER(C.c_double)]
        _lib = L
    return _lib


def c_config(cfg: ModelConfig) -> SdModelConfig:
    return SdModelConfig({"gpt2": 0, "llama": 1}[cfg.arch], {"f32": 0, "bf16": 1}[cfg.dtype], cfg.n_layer, cfg.d_model,
                         cfg.n_head, cfg.n_kv_head, cfg.d_ff, cfg.vocab, cfg.n_ctx, int(cfg.bidirectional),
                         cfg.norm_eps, cfg.rope_theta)


def sd_vocab_pad(vocab: int) -> int:
    return lib().sd_vocab_pad(vocab)


def sd_weight_layout(cfg: ModelConfig) -> List[Tuple[str, int, int, int, int]]:
    """[(name, rows, cols, elem_bytes, offset)] in storage order."""
    L, cc = lib(), c_config(cfg)
    out = []
    for i in range(L.sd_weight_count(C.byref(cc))):
        name = C.create_string_buffer(64)
        rows, cols, eb, off = C.c_int64(), C.c_int64(), C.c_int32(), C.c_int64()
        rc = L.sd_weight_desc(C.byref(cc), i, name, 64, C.byref(rows), C.byref(cols), C.byref(eb), C.byref(off))
        if rc:
            raise SdError(rc, "sd_weight_desc")
        out.append((name.value.decode(), rows.value, cols.value, eb.value, off.value))
    return out


def sd_weight_bytes(cfg: ModelConfig) -> int:
    cc = c_config(cfg)
    return lib().sd_weight_bytes(C.byref(cc))


def sd_workspace_bytes(target: ModelConfig, drafter: ModelConfig, max_batch: int, gamma_max: int) -> int:
    ct, cd = c_config(target), c_config(drafter)
    return lib().sd_workspace_bytes(C.byref(ct), C.byref(cd), max_batch, gamma_max)


def pack_weights(cfg: ModelConfig, weights: Dict[str, np.ndarray], threads: int = 8) -> np.ndarray:
    """Host image (uint8) of the flat weight buffer in the library's layout."""
    buf = np.zeros(sd_weight_bytes(cfg), dtype=np.uint8)

    def put(entry):
        name, rows, cols, eb, off = entry
        w = np.ascontiguousarray(weights[name], dtype=np.float32).reshape(rows, cols)
        if eb == 4:
            raw = w.view(np.uint8).reshape(-1)
        else:   # bf16 storage: values are already bf16-representable; keep the upper 16 bits
            bits = w.view(np.uint32)
            assert not (bits & 0xFFFF).any(), f"{name}: value not representable in bf16"
            raw = (bits >> 16).astype(np.uint16).view(np.uint8).reshape(-1)
        buf[off:off + raw.size] = raw

    layout = sd_weight_layout(cfg)
    if threads <= 1 or len(layout) < 8:
        for e in layout:
            put(e)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(put, layout))
    return buf


def _ip(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _ragged(seqs: Sequence[Sequence[int]]):
    lens = np.array([len(s) for s in seqs], dtype=np.int32)
    flat = np.ascontiguousarray(np.concatenate([np.asarray(s, dtype=np.int32) for s in seqs]))
    return flat, lens


class SpecDiff:
    """Owns the device buffers (through torch) and a library handle."""

    def __init__(self, target: ModelConfig, drafter: ModelConfig, target_w: Dict[str, np.ndarray],
                 drafter_w: Dict[str, np.ndarray], max_batch: int = 1, gamma_max: int = 64, device: str = "cuda:0",
                 device_weights=None):
        """target_w / drafter_w: host tensors by name (packed and uploaded here), or -- device_weights = (target buffer,
        drafter buffer), uint8 device tensors already in the library's layout (pack_weights) -- None."""
        import torch
        self.torch = torch
        self.target, self.drafter = target, drafter
        self.max_batch, self.gamma_max = max_batch, gamma_max
        self.device = torch.device(device)
        self.ld = sd_vocab_pad(target.vocab)
        if device_weights is not None:
            self.tw, self.dw = device_weights
            assert self.tw.numel() == sd_weight_bytes(target) and self.dw.numel() == sd_weight_bytes(drafter)
        else:
            self.tw = torch.from_numpy(pack_weights(target, target_w)).to(self.device)
            self.dw = torch.from_numpy(pack_weights(drafter, drafter_w)).to(self.device)
        nbytes = sd_workspace_bytes(target, drafter, max_batch, gamma_max)
        if nbytes <= 0:
            raise SdError(1, "sd_workspace_bytes", "configuration rejected")
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8, device=self.device)
        # A stream of its own (default priority): launch sequences are captured into HIP graphs,
        # which the legacy default stream does not allow.
        self.stream = torch.cuda.Stream(self.device)
        torch.cuda.synchronize(self.device)       # weights and workspace are in place before the first call
        self._ct, self._cd = c_config(target), c_config(drafter)
        h = C.c_void_p()
        rc = lib().sd_create(C.byref(self._ct), C.byref(self._cd), self.tw.data_ptr(), self.dw.data_ptr(), max_batch,
                             gamma_max, self.workspace.data_ptr(), nbytes, self.stream.cuda_stream, C.byref(h))
        if rc:
            raise SdError(rc, "sd_create", lib().sd_last_error(None).decode())
        self.h = h
        self._destroy = lib().sd_destroy          # module globals may be gone when __del__ runs at interpreter exit

    def close(self):
        if getattr(self, "h", None):
            self._destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def _check(self, rc: int, where: str):
        if rc:
            raise SdError(rc, where, lib().sd_last_error(self.h).decode())

    def _view(self, ptr: int, rows: int):
        """fp32 [rows, ld] view of library-owned device memory inside the workspace."""
        off = ptr - self.workspace.data_ptr()
        assert 0 <= off and off + rows * self.ld * 4 <= self.workspace.numel()
        return self.workspace[off:off + rows * self.ld * 4].view(self.torch.float32).view(rows, self.ld)

    def sd_set_graph_replay(self, enable: bool):
        self._check(lib().sd_set_graph_replay(self.h, int(enable)), "sd_set_graph_replay")

    def sd_graph_stats(self):
        """-> dict(replays, eager_after_failure, failures, captured, error)."""
        r, e, f, c = C.c_int64(), C.c_int64(), C.c_int32(), C.c_int32()
        self._check(lib().sd_graph_stats(self.h, C.byref(r), C.byref(e), C.byref(f), C.byref(c)), "sd_graph_stats")
        return dict(replays=r.value, eager_after_failure=e.value, failures=f.value, captured=c.value,
                    error=lib().sd_graph_error(self.h).decode())

    def sd_profile_begin(self):
        self._check(lib().sd_profile_begin(self.h), "sd_profile_begin")

    def sd_profile_end(self):
        """-> [dict(name, launches, ms, bytes, flops)] accumulated since sd_profile_begin."""
        self._check(lib().sd_profile_end(self.h), "sd_profile_end")
        out = []
        for i in range(lib().sd_profile_count(self.h)):
            name = C.create_string_buffer(128)
            n, ms, by, fl = C.c_int64(), C.c_double(), C.c_double(), C.c_double()
            self._check(lib().sd_profile_entry(self.h, i, name, 128, C.byref(n), C.byref(ms), C.byref(by), C.byref(fl)),
                        "sd_profile_entry")
            out.append(dict(name=name.value.decode(), launches=n.value, ms=ms.value, bytes=by.value, flops=fl.value))
        return out

    def sd_prefill(self, prefixes):
        flat, lens = _ragged(prefixes)
        self._check(lib().sd_prefill(self.h, len(lens), _ip(flat), _ip(lens)), "sd_prefill")

    def sd_draft(self, prefixes, gamma: int, T: int, seed: int):
        """-> (draft int32 [B, gamma], qtok fp32 [B, gamma], q device tensor fp32 [B*gamma, ld])."""
        flat, lens = _ragged(prefixes)
        B = len(lens)
        draft = np.zeros((B, gamma), dtype=np.int32)
        qtok = np.zeros((B, gamma), dtype=np.float32)
        qp = C.c_void_p()
        self._check(lib().sd_draft(self.h, B, _ip(flat), _ip(lens), gamma, T, seed, _ip(draft),
                                   qtok.ctypes.data_as(C.POINTER(C.c_float)), C.byref(qp)), "sd_draft")
        return draft, qtok, (self._view(qp.value, B * gamma) if qp.value else None)      # no q at temperature 0

    def sd_verify(self, prefixes, draft: np.ndarray, q_dev, seed: int):
        """-> (n_accepted int32 [B], token int32 [B])."""
        flat, lens = _ragged(prefixes)
        B = len(lens)
        draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(B, -1)
        n = np.zeros(B, dtype=np.int32)
        tok = np.zeros(B, dtype=np.int32)
        self._check(lib().sd_verify(self.h, B, _ip(flat), _ip(lens), draft.shape[1], _ip(draft),
                                    q_dev.data_ptr() if q_dev is not None else None, seed, _ip(n), _ip(tok)), "sd_verify")
        return n, tok

    def sd_round(self, prefixes, gamma: int, T: int, seed: int):
        """-> (draft [B, gamma], n_accepted [B], token [B])."""
        flat, lens = _ragged(prefixes)
        return self.sd_round_flat(flat, lens, gamma, T, seed)

    def sd_round_flat(self, flat: np.ndarray, lens: np.ndarray, gamma: int, T: int, seed: int):
        B = len(lens)
        draft = np.zeros((B, gamma), dtype=np.int32)
        n = np.zeros(B, dtype=np.int32)
        tok = np.zeros(B, dtype=np.int32)
        self._check(lib().sd_round(self.h, B, _ip(flat), _ip(lens), gamma, T, seed, _ip(draft), _ip(n), _ip(tok)), "sd_round")
        return draft, n, tok

    # ---- standard speculative decoding: an autoregressive drafter beside the diffusion drafter
    def sd_sps_attach(self, cfg: ModelConfig, weights: Dict[str, np.ndarray] = None, device_weights=None):
        torch = self.torch
        self.sps = cfg
        self._cs = c_config(cfg)
        self.sw = device_weights if device_weights is not None else torch.from_numpy(pack_weights(cfg, weights)).to(self.device)
        nbytes = lib().sd_sps_workspace_bytes(self.h, C.byref(self._cs))
        if nbytes <= 0:
            raise SdError(1, "sd_sps_workspace_bytes", "configuration rejected")
        self.sps_workspace = torch.zeros(nbytes, dtype=torch.uint8, device=self.device)
        torch.cuda.synchronize(self.device)
        self._check(lib().sd_sps_attach(self.h, C.byref(self._cs), self.sw.data_ptr(), self.sps_workspace.data_ptr(), nbytes), "sd_sps_attach")

    def sd_sps_draft(self, prefixes, gamma: int, seed: int):
        """-> (draft int32 [B, gamma], qtok fp32 [B, gamma], q device tensor fp32 [B*gamma, ld] or None)."""
        flat, lens = _ragged(prefixes)
        B = len(lens)
        draft = np.zeros((B, gamma), dtype=np.int32)
        qtok = np.zeros((B, gamma), dtype=np.float32)
        qp = C.c_void_p()
        self._check(lib().sd_sps_draft(self.h, B, _ip(flat), _ip(lens), gamma, seed, _ip(draft),
                                       qtok.ctypes.data_as(C.POINTER(C.c_float)), C.byref(qp)), "sd_sps_draft")
        return draft, qtok, (self._view(qp.value, B * gamma) if qp.value else None)

    def sd_sps_round(self, prefixes, gamma: int, seed: int):
        flat, lens = _ragged(prefixes)
        return self.sd_sps_round_flat(flat, lens, gamma, seed)

    def sd_sps_round_flat(self, flat: np.ndarray, lens: np.ndarray, gamma: int, seed: int):
        B = len(lens)
        draft = np.zeros((B, gamma), dtype=np.int32)
        n = np.zeros(B, dtype=np.int32)
        tok = np.zeros(B, dtype=np.int32)
        self._check(lib().sd_sps_round(self.h, B, _ip(flat), _ip(lens), gamma, seed, _ip(draft), _ip(n), _ip(tok)), "sd_sps_round")
        return draft, n, tok

    def sd_sps_logits(self, sequences):
        """Next-token logits of the autoregressive drafter after each sequence -> device fp32 [B, ld]."""
        flat, lens = _ragged(sequences)
        p = C.c_void_p()
        self._check(lib().sd_sps_logits(self.h, len(lens), _ip(flat), _ip(lens), C.byref(p)), "sd_sps_logits")
        return self._view(p.value, len(lens))

    def generate_hybrid(self, prefixes, n_new: int, gamma_sps: int, gamma: int, T: int, seed: int, n_init: int):
        """Sequence initialisation: rounds of sd_sps_round until every sequence has n_init new tokens, then rounds of
        sd_round, until n_new; round i uses seed + i; sd_commit after every round.
        -> (new tokens per sequence, accepted counts [rounds, B], number of SpS rounds)."""
        seqs = [list(int(t) for t in p) for p in prefixes]
        start = [len(s) for s in seqs]
        accepted = []
        rnd = sps_rounds = 0
        while min(len(s) - l for s, l in zip(seqs, start)) < n_new:
            if min(len(s) - l for s, l in zip(seqs, start)) < n_init:
                draft, n, tok = self.sd_sps_round(seqs, gamma_sps, seed + rnd)
                sps_rounds += 1
            else:
                draft, n, tok = self.sd_round(seqs, gamma, T, seed + rnd)
            self.sd_commit(n)
            for b, s in enumerate(seqs):
                s.extend(int(t) for t in draft[b, :n[b]])
                s.append(int(tok[b]))
            accepted.append(n.copy())
            rnd += 1
        return [np.array(s[l:], dtype=np.int64) for s, l in zip(seqs, start)], accepted, sps_rounds

    def sd_commit(self, n_accepted):
        n = np.ascontiguousarray(n_accepted, dtype=np.int32)
        self._check(lib().sd_commit(self.h, len(n), _ip(n)), "sd_commit")

    def sd_set_step_skipping(self, enable: bool):
        self._check(lib().sd_set_step_skipping(self.h, 1 if enable else 0), "sd_set_step_skipping")

    def sd_steps_run(self) -> int:
        return int(lib().sd_steps_run(self.h))

    def sd_set_greedy(self, enable: bool):
        self._check(lib().sd_set_greedy(self.h, 1 if enable else 0), "sd_set_greedy")

    def generate(self, prefixes, n_new: int, gamma: int, T: int, seed: int):
        """Rounds of sd_round + sd_commit until every sequence has at least n_new new tokens; round i uses
        seed + i.  -> (list of new-token arrays, list of per-round accepted counts [rounds, B])."""
        seqs = [list(int(t) for t in p) for p in prefixes]
        start = [len(s) for s in seqs]
        accepted = []
        rnd = 0
        while min(len(s) - l for s, l in zip(seqs, start)) < n_new:
            draft, n, tok = self.sd_round(seqs, gamma, T, seed + rnd)
            self.sd_commit(n)
            for b, s in enumerate(seqs):
                s.extend(int(t) for t in draft[b, :n[b]])
                s.append(int(tok[b]))
            accepted.append(n.copy())
            rnd += 1
        return [np.array(s[l:], dtype=np.int64) for s, l in zip(seqs, start)], np.array(accepted)

    def sd_drafter_logits(self, sequences, gamma: int, step: int, T: int):
        """sequences: prefix o block per batch element (mask id = vocab).  -> device fp32 [B*gamma, ld]."""
        flat, lens = _ragged(sequences)
        p = C.c_void_p()
        self._check(lib().sd_drafter_logits(self.h, len(lens), _ip(flat), _ip(lens), gamma, step, T, C.byref(p)),
                    "sd_drafter_logits")
        return self._view(p.value, len(lens) * gamma)

    def sd_target_logits(self, prefixes, draft: np.ndarray):
        flat, lens = _ragged(prefixes)
        B = len(lens)
        draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(B, -1)
        p = C.c_void_p()
        self._check(lib().sd_target_logits(self.h, B, _ip(flat), _ip(lens), draft.shape[1], _ip(draft), C.byref(p)),
                    "sd_target_logits")
        return self._view(p.value, B * (draft.shape[1] + 1))


# ---- stand-alone kernels on torch device tensors --------------------------------------------------
def _stream_ptr(t):
    import torch
    return torch.cuda.current_stream(t.device).cuda_stream


def sd_sampling_scratch_bytes(rows: int, vocab: int) -> int:
    return lib().sd_sampling_scratch_bytes(rows, vocab)


def sd_unmask_sample(logits, batch: int, gamma: int, vocab: int, step: int, seed: int, z, q, qtok):
    """In place on device tensors: logits fp32 [B*gamma, ld], z int32 [B*gamma], q fp32 [B*gamma, ld], qtok fp32."""
    import torch
    nb = sd_sampling_scratch_bytes(batch * (gamma + 1), vocab)
    scratch = torch.empty(nb, dtype=torch.uint8, device=logits.device)
    rc = lib().sd_unmask_sample(logits.data_ptr(), batch, gamma, vocab, step, seed, z.data_ptr(), q.data_ptr(),
                                qtok.data_ptr(), scratch.data_ptr(), nb, _stream_ptr(logits))
    if rc:
        raise SdError(rc, "sd_unmask_sample")
    torch.cuda.synchronize(logits.device)


def sd_accept_resample(p_logits, q, draft, batch: int, gamma: int, vocab: int, seed: int):
    """-> (n_accepted, token) int32 device tensors [B]."""
    import torch
    nb = sd_sampling_scratch_bytes(batch * (gamma + 1), vocab)
    scratch = torch.empty(nb, dtype=torch.uint8, device=p_logits.device)
    n = torch.zeros(batch, dtype=torch.int32, device=p_logits.device)
    tok = torch.zeros(batch, dtype=torch.int32, device=p_logits.device)
    rc = lib().sd_accept_resample(p_logits.data_ptr(), q.data_ptr(), draft.data_ptr(), batch, gamma, vocab, seed,
                                  n.data_ptr(), tok.data_ptr(), scratch.data_ptr(), nb, _stream_ptr(p_logits))
    if rc:
        raise SdError(rc, "sd_accept_resample")
    torch.cuda.synchronize(p_logits.device)
    return n, tok


def sd_accept_resample_static(p_logits, q, draft, batch: int, gamma: int, vocab: int, seed: int, n, tok):
    """The same on the library's fixed scratch buffer; n, tok: caller's int32 device tensors [B].  Allocates nothing."""
    import torch
    rc = lib().sd_accept_resample_static(p_logits.data_ptr(), q.data_ptr(), draft.data_ptr(), batch, gamma, vocab, seed,
                                         n.data_ptr(), tok.data_ptr(), _stream_ptr(p_logits))
    if rc:
        raise SdError(rc, "sd_accept_resample_static", lib().sd_last_error(None).decode())
    torch.cuda.synchronize(p_logits.device)


_split_ws = {}


def split_workspace(device, part_bytes: int = 64 << 20):
    """Zero-filled device workspace for the contractions that split K over workgroups (one per device)."""
    import torch
    key = str(device)
    if key not in _split_ws:
        _split_ws[key] = torch.zeros(int(lib().sd_linear_split_ticket_bytes()) + part_bytes, dtype=torch.uint8, device=device)
    return _split_ws[key]


def sd_linear(dtype: str, x, w, bias, y, epilogue: int, split: bool = True):
    """y = epilogue(x w^T + bias) on device tensors; see specdiff.h."""
    import torch
    m, k = x.shape
    n = w.shape[0]
    ws = split_workspace(x.device) if split else None
    rc = lib().sd_linear({"f32": 0, "bf16": 1}[dtype], x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                         y.data_ptr(), m, n, k, y.stride(0), epilogue, ws.data_ptr() if split else None,
                         ws.numel() if split else 0, _stream_ptr(x))
    if rc:
        raise SdError(rc, "sd_linear")
    torch.cuda.synchronize(x.device)


def sd_norm_linear(norm_kind: int, h, w, gain, beta, bias, y, epilogue: int, eps: float, split: bool = True):
    """y = epilogue(w norm(h) + bias) with the norm folded into the contraction; device tensors."""
    import torch
    m, k = h.shape
    n = w.shape[0]
    scratch = torch.empty(int(lib().sd_norm_linear_scratch_floats(m, n, k)), dtype=torch.float32, device=h.device)
    ws = split_workspace(h.device) if split else None
    rc = lib().sd_norm_linear(norm_kind, h.data_ptr(), w.data_ptr(), gain.data_ptr(), beta.data_ptr() if beta is not None else None,
                              bias.data_ptr() if bias is not None else None, y.data_ptr(), m, n, k, y.stride(0), epilogue, eps,
                              scratch.data_ptr(), ws.data_ptr() if split else None, ws.numel() if split else 0, _stream_ptr(h))
    if rc:
        raise SdError(rc, "sd_norm_linear")
    torch.cuda.synchronize(h.device)


def sd_linear_resid_norm(x, w, bias, y, gain, split: bool = True):
    """y += x w^T + bias (fp32, in place); returns (xg bf16 [m, n], stats fp32 [m, ceil(n/32), 2]); see specdiff.h."""
    import torch
    m, k = x.shape
    n = w.shape[0]
    xg = torch.zeros(m, n, dtype=torch.bfloat16, device=x.device)
    stats = torch.zeros(m, (n + 31) // 32, 2, dtype=torch.float32, device=x.device)
    ws = split_workspace(x.device) if split else None
    rc = lib().sd_linear_resid_norm(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None, y.data_ptr(),
                                    gain.data_ptr(), xg.data_ptr(), stats.data_ptr(), m, n, k,
                                    ws.data_ptr() if split else None, ws.numel() if split else 0, _stream_ptr(x))
    if rc:
        raise SdError(rc, "sd_linear_resid_norm")
    torch.cuda.synchronize(x.device)
    return xg, stats
