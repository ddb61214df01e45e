"""Convenience driver around the C ABI for tests and the benchmark: owns the pinned
host blobs, the device buffers a step needs, and issues the calls in the order of
Alg. 1 (refresh every tau steps, then the step).  No arithmetic happens here."""
from __future__ import annotations

import concurrent.futures
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as tb

ExpertBits = Callable[[int], Tuple[np.ndarray, np.ndarray, np.ndarray]]


class TideSession:
    def __init__(self, d: int, E: int, k: int, I: int, n_shared: int, capacity: int, max_tokens: int,
                 gating: int, bias_mode: int, n_layers: int = 1, device: str = "cuda:0", resident_p12: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("TideSession needs a GPU; there is no CPU path")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.resident_p12 = bool(resident_p12)
        self.cfg = tb.make_config(d, E, k, I, n_shared, n_layers, capacity, max_tokens, gating, bias_mode,
                                  tb.TIDE_RESIDENT_P12 if resident_p12 else tb.TIDE_RESIDENT_BF16)
        self.comp_blobs = {}
        self.d, self.E, self.k, self.I, self.n_shared, self.C = d, E, k, I, n_shared, capacity
        self.max_tokens, self.n_layers = max_tokens, n_layers
        self.blob_bytes = tb.tide_expert_blob_bytes(self.cfg)
        self.ctx = tb.tide_create(self.cfg)
        self.host_blobs: List[Optional[torch.Tensor]] = [None] * n_layers
        P = max_tokens * k
        self.out = torch.empty((max_tokens, d), dtype=torch.float32, device=self.device)
        self.miss = torch.empty((max(P, 1), 3), dtype=torch.int32, device=self.device)
        self.n_miss = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.topk_idx = torch.empty((max_tokens, k), dtype=torch.int32, device=self.device)
        self.topk_w = torch.empty((max_tokens, k), dtype=torch.float32, device=self.device)
        self.router_w: List[Optional[torch.Tensor]] = [None] * n_layers
        self.router_b: List[Optional[torch.Tensor]] = [None] * n_layers

    # ------------------------------------------------------------------ set-up
    def pack_layer(self, expert_bits: ExpertBits, workers: int = 8):
        """Packs a layer's E routed experts into one pinned tensor [E, blob_bytes] and the shared
        expert (if any) into a host array.  The result can be attached to several sessions."""
        blobs = torch.empty((self.E, self.blob_bytes), dtype=torch.uint8, pin_memory=True)
        np_blobs = blobs.numpy()

        def one(e: int) -> None:
            wg, wu, wd = expert_bits(e)
            tb.tide_pack_expert(self.cfg, wg, wu, wd, np_blobs[e])

        with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(one, range(self.E)))
        sh = None
        if self.n_shared:
            sh = np.empty(self.blob_bytes, dtype=np.uint8)
            tb.tide_pack_expert(self.cfg, *expert_bits(self.E), sh)
        return blobs, sh

    def compress_layer(self, layer: int, workers: int = 8, comp: Optional[torch.Tensor] = None) -> None:
        """Builds the 12-bit form of the layer's registered blobs in pinned memory (or takes one built earlier for the
        same blobs) and registers it: the source of the layer's refresh copies (3/4 of the bytes over the host link)
        and, in a session with 12-bit slots, what the slots hold."""
        comp_bytes = tb.tide_compressed_blob_bytes(self.cfg)
        if comp is None:
            comp = torch.empty((self.E, comp_bytes), dtype=torch.uint8, pin_memory=True)
            raw, out = self.host_blobs[layer].numpy(), comp.numpy()
            with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as ex:
                list(ex.map(lambda e: tb.tide_compress_expert(self.cfg, raw[e], out[e]), range(self.E)))
        assert tuple(comp.shape) == (self.E, comp_bytes) and comp.is_pinned()
        self.comp_blobs[layer] = comp
        tb.tide_register_compressed(self.ctx, layer, comp, comp_bytes)

    def load_layer(self, layer: int, expert_bits: Optional[ExpertBits], router_w: np.ndarray,
                   router_bias: Optional[np.ndarray], resident: Sequence[int], workers: int = 8, packed=None,
                   comp: Optional[torch.Tensor] = None) -> None:
        blobs, sh = packed if packed is not None else self.pack_layer(expert_bits, workers)
        assert tuple(blobs.shape) == (self.E, self.blob_bytes) and blobs.is_pinned()
        self.host_blobs[layer] = blobs
        tb.tide_register_experts(self.ctx, layer, blobs, self.blob_bytes)
        if self.resident_p12 or comp is not None:        # 12-bit slots are filled from the compressed blobs
            self.compress_layer(layer, workers, comp)
        if self.n_shared:
            tb.tide_set_shared(self.ctx, layer, sh)
        tb.tide_set_resident(self.ctx, layer, resident)
        self.router_w[layer] = torch.from_numpy(np.ascontiguousarray(router_w, dtype=np.float32)).to(self.device)
        self.router_b[layer] = (None if router_bias is None else
                                torch.from_numpy(np.ascontiguousarray(router_bias, dtype=np.float32)).to(self.device))

    def to_device_bf16(self, bits: np.ndarray) -> torch.Tensor:
        """uint16 bf16 bit patterns -> device tensor holding the same bits."""
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(self.device)

    # ------------------------------------------------------------------ calls
    def step(self, layer: int, hidden_dev: torch.Tensor, n_tokens: Optional[int] = None, miss_cap: Optional[int] = None,
             want_topk: bool = True) -> None:
        n = hidden_dev.shape[0] if n_tokens is None else n_tokens
        cap = n * self.k if miss_cap is None else miss_cap
        tb.tide_moe_step(self.ctx, layer, hidden_dev, n, self.router_w[layer], self.router_b[layer], self.out,
                         self.miss, cap, self.n_miss, self.topk_idx if want_topk else None,
                         self.topk_w if want_topk else None, torch.cuda.current_stream())

    def stack_step(self, hidden_devs, first_layer: int = 0, miss_cap: Optional[int] = None) -> None:
        """One denoise step of the independent layers first_layer .. first_layer + len(hidden_devs) - 1 through
        tide_moe_stack_step.  Results per layer in self.stack_out / stack_miss / stack_n_miss (made on first use)."""
        n_layers = len(hidden_devs)
        n = hidden_devs[0].shape[0]
        if not hasattr(self, "stack_out"):
            P = self.max_tokens * self.k
            self.stack_out = [torch.empty((self.max_tokens, self.d), dtype=torch.float32, device=self.device) for _ in range(self.n_layers)]
            self.stack_miss = [torch.empty((max(P, 1), 3), dtype=torch.int32, device=self.device) for _ in range(self.n_layers)]
            self.stack_n_miss = [torch.zeros(1, dtype=torch.int32, device=self.device) for _ in range(self.n_layers)]
        sl = slice(first_layer, first_layer + n_layers)
        cap = n * self.k if miss_cap is None else miss_cap
        tb.tide_moe_stack_step(self.ctx, first_layer, hidden_devs, n, self.router_w[sl], self.router_b[sl], self.stack_out[sl],
                               self.stack_miss[sl], cap, self.stack_n_miss[sl], torch.cuda.current_stream())

    def step_routed(self, layer: int, hidden_dev: torch.Tensor, idx_dev: torch.Tensor, w_dev: torch.Tensor,
                    miss_cap: Optional[int] = None) -> None:
        n = hidden_dev.shape[0]
        cap = n * self.k if miss_cap is None else miss_cap
        tb.tide_moe_step_routed(self.ctx, layer, hidden_dev, n, idx_dev, w_dev, self.out, self.miss, cap, self.n_miss,
                                torch.cuda.current_stream())

    def apply_misses(self, layer: int, hidden_dev: torch.Tensor, miss_cap: Optional[int] = None) -> None:
        """Adds the last step's misses (evaluated from the host-resident blobs) to self.out."""
        n = hidden_dev.shape[0]
        cap = n * self.k if miss_cap is None else miss_cap
        tb.tide_moe_apply_misses(self.ctx, layer, hidden_dev, n, self.miss, cap, self.n_miss, self.out,
                                 torch.cuda.current_stream())

    def host_experts(self, n_threads: int) -> None:
        tb.tide_host_experts(self.ctx, n_threads)

    def apply_misses_host(self, layer: int, hidden_dev: torch.Tensor, miss_cap: Optional[int] = None) -> None:
        """Adds the last step's misses, evaluated by the host workers, to self.out."""
        n = hidden_dev.shape[0]
        cap = n * self.k if miss_cap is None else miss_cap
        tb.tide_moe_apply_misses_host(self.ctx, layer, hidden_dev, n, self.miss, cap, self.n_miss, self.out,
                                      torch.cuda.current_stream())

    def results(self, n_tokens: int):
        """(out[n,d] fp32, idx[n,k], w[n,k], miss list of (token, expert, weight)) on the host."""
        torch.cuda.synchronize()
        out = self.out[:n_tokens].cpu().numpy()
        idx = self.topk_idx[:n_tokens].cpu().numpy()
        w = self.topk_w[:n_tokens].cpu().numpy()
        n_miss = int(self.n_miss.item())
        raw = np.ascontiguousarray(self.miss[:min(n_miss, self.miss.shape[0])].cpu().numpy())
        wts = raw[:, 2].copy().view(np.float32)
        miss = [(int(r[0]), int(r[1]), float(x)) for r, x in zip(raw, wts)]
        return out, idx, w, miss, n_miss

    def stats(self, layer: int, reset: bool = False) -> np.ndarray:
        return tb.tide_interval_stats(self.ctx, layer, self.E, reset, torch.cuda.current_stream())

    def refresh(self, layer: int, capacity: Optional[int] = None, counts: Optional[np.ndarray] = None,
                reset_counts: bool = True, deferred: bool = False):
        return tb.tide_refresh(self.ctx, layer, self.C, self.C if capacity is None else capacity, counts, reset_counts,
                               torch.cuda.current_stream(), deferred=deferred)

    def refresh_async(self, layer: int, capacity: Optional[int] = None, counts: Optional[np.ndarray] = None,
                      reset_counts: bool = True) -> None:
        tb.tide_refresh_async(self.ctx, layer, self.C if capacity is None else capacity, counts, reset_counts,
                              torch.cuda.current_stream())

    def refresh_result(self, layer: int):
        return tb.tide_refresh_result(self.ctx, layer, self.C)

    def commit(self, layer: int) -> None:
        tb.tide_commit(self.ctx, layer, torch.cuda.current_stream())

    def table(self, layer: int) -> np.ndarray:
        return tb.tide_get_table(self.ctx, layer, self.E, torch.cuda.current_stream())

    def read_slot(self, layer: int, slot: int) -> np.ndarray:
        return tb.tide_read_slot(self.ctx, layer, slot, self.blob_bytes)

    def close(self) -> None:
        if self.ctx:
            torch.cuda.synchronize()
            tb.tide_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
