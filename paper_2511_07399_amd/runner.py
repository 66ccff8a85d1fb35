"""Device-side setup of a workload: weights in HBM, the C structs that point at them, the rolling
cache, the text K/V and the workspace, plus thin methods that call the library.

Plumbing only: tensors are drawn by ``workloads`` and every step of the path runs in libsdv2.
"""

import numpy as np
import torch

from . import binding, workloads as wk


class DeviceModel:
    """Device tensors, C structs, cache, text K/V and workspace of one workload on one GPU."""

    def __init__(self, wl, base_seed=0, device="cuda:0", n_layers=None, n_streams=None, weight_device="cpu",
                 sink_tokens=None, window_tokens=None, edit=None):
        """weight_device: where the seeded generators run ("cpu" values are the ones a host-side checker can
        redraw; a CUDA generator draws other values from the same seed), or a callable layer -> device.
        edit: optional callable (tensors, layer) applied to each layer's freshly drawn tensors, in place, before
        they are uploaded (tests use it to rescale gates or to switch a branch off)."""
        binding.load_library()
        self.wl = wl
        self.device = torch.device(device)
        self.N = wl.N if n_layers is None else n_layers
        self.n_streams = wl.B if n_streams is None else n_streams
        self.S = wl.S if sink_tokens is None else sink_tokens
        self.W = wl.W if window_tokens is None else window_tokens
        self.cfg = binding.model_cfg(wl.C, wl.H, wl.F, wl.grid_h, wl.grid_w, wl.L_t, self.N, wl.t_dim)
        self.layers = []
        self.bw_array = (binding.BlockWeights * self.N)()
        for layer in range(self.N):
            wdev = weight_device(layer) if callable(weight_device) else weight_device
            w = wk.block_weights(wl, layer, base_seed, device=wdev)
            if edit is not None:
                edit(w, layer)
            t = {k: v.to(self.device) for k, v in w.items()}
            t["W_qkv"] = torch.cat([t.pop("W_q"), t.pop("W_k"), t.pop("W_v")], 0).contiguous()
            t["b_qkv"] = torch.cat([t.pop("b_q"), t.pop("b_k"), t.pop("b_v")], 0).contiguous()
            self.layers.append(t)
            self.bw_array[layer] = binding.block_weights(t)
        mw = wk.model_weights(wl, base_seed, device="cpu" if callable(weight_device) else weight_device)
        self.mw_t = {k: v.to(self.device) for k, v in mw.items()}
        self.mw = binding.model_weights(self.mw_t, self.bw_array)
        # cache: poisoned with 0xFF bytes (bf16 NaN, id -1) so that a read of an unfilled slot shows up
        self.ccfg = binding.cache_cfg(self.N, self.n_streams, wl.H, wl.P, self.S, self.W)
        self.cache_storage = torch.full((binding.kv_cache_bytes(self.ccfg),), 0xFF, dtype=torch.uint8, device=self.device)
        self.cache = binding.kv_cache_init(self.ccfg, self.cache_storage)
        # text K/V per (layer, stream)
        tkv = binding.text_kv_bytes(self.cfg)
        self.kt = [[torch.full((tkv,), 0xFF, dtype=torch.uint8, device=self.device) for _ in range(self.n_streams)]
                   for _ in range(self.N)]
        self.vtt = [[torch.full((tkv,), 0xFF, dtype=torch.uint8, device=self.device) for _ in range(self.n_streams)]
                    for _ in range(self.N)]
        tws = torch.empty(binding.text_kv_workspace_bytes(self.cfg), dtype=torch.uint8, device=self.device)
        for s in range(self.n_streams):
            ctx = wk.text_context(wl, s, base_seed).to(self.device, torch.bfloat16)
            for layer in range(self.N):
                binding.text_kv_prepare(self.cfg, self.bw_array[layer], ctx, self.kt[layer][s], self.vtt[layer][s], tws)
        self._ws = {}

    def workspace(self, B, L):
        key = (B, L)
        if key not in self._ws:
            self._ws[key] = torch.empty(binding.denoise_workspace_bytes(self.cfg, B, L), dtype=torch.uint8,
                                        device=self.device)
        return self._ws[key]

    def conditioning(self, B, timesteps=None, tvec=None):
        e0 = torch.empty(B, 6, self.wl.C, dtype=torch.float32, device=self.device)
        ws = torch.empty(max(binding.conditioning_workspace_bytes(self.cfg, B), 256), dtype=torch.uint8, device=self.device)
        binding.conditioning(self.cfg, self.mw, B, e0, ws, timesteps=timesteps, tvec=tvec)
        return e0

    def block(self, layer, x, e0, descs):
        """x: fp32 [B, L, C] device tensor, updated in place.  descs: list of (stream, frame_pos0, n_frames, advance)."""
        B, L, _ = x.shape
        pick = lambda d: min(max(d[0], 0), self.n_streams - 1)     # bad ids still reach the library
        kt = [self.kt[layer][pick(d)] for d in descs]
        vtt = [self.vtt[layer][pick(d)] for d in descs]
        binding.dit_block_forward(self.cfg, self.bw_array[layer], self.cache, layer, x, e0, kt, vtt,
                                  binding.chunk_descs(descs), self.workspace(B, L))

    def denoise(self, x, descs, timesteps=None, tvec=None):
        B, L, _ = x.shape
        kt = binding.ptr_array([self.kt[layer][d[0]] for layer in range(self.N) for d in descs])
        vtt = binding.ptr_array([self.vtt[layer][d[0]] for layer in range(self.N) for d in descs])
        binding.denoise_step(self.cfg, self.mw, self.cache, x, kt, vtt, binding.chunk_descs(descs),
                             self.workspace(B, L), timesteps=timesteps, tvec=tvec)

    def io(self, base_seed=0):
        """Patch-embedding and output-head weights in HBM and the struct that points at them (made on first use)."""
        if not hasattr(self, "_io"):
            self.io_t = {k: v.to(self.device) for k, v in wk.io_weights(self.wl, base_seed).items()}
            self._io = binding.io_weights(self.io_t)
        return self._io

    def denoise_latents(self, z, descs, sigmas, sigmas_next, eps_next=None, x0=None):
        """z: fp32 [B, 16, F, 2 grid_h, 2 grid_w] device tensor, updated in place to the next step's input."""
        B, L = z.shape[0], z.shape[2] * self.wl.grid_h * self.wl.grid_w
        pick = lambda d: min(max(d[0], 0), self.n_streams - 1)     # bad ids still reach the library
        kt = binding.ptr_array([self.kt[layer][pick(d)] for layer in range(self.N) for d in descs])
        vtt = binding.ptr_array([self.vtt[layer][pick(d)] for layer in range(self.N) for d in descs])
        key = ("latents", B, L)
        if key not in self._ws:
            self._ws[key] = torch.empty(binding.denoise_latents_workspace_bytes(self.cfg, B, L), dtype=torch.uint8,
                                        device=self.device)
        binding.denoise_latents_step(self.cfg, self.mw, self.io(), self.cache, z, eps_next, x0, sigmas, sigmas_next,
                                     kt, vtt, binding.chunk_descs(descs), self._ws[key])

    def graph(self, x, stream_ids, n_frames):
        """Records sdv2_denoise_step on the fp32 [B, L, C] tensor x for these streams; returns the handle (the
        workspace and the descriptor buffer stay alive in this object)."""
        B, L, _ = x.shape
        kt = binding.ptr_array([self.kt[layer][s] for layer in range(self.N) for s in stream_ids])
        vtt = binding.ptr_array([self.vtt[layer][s] for layer in range(self.N) for s in stream_ids])
        state = torch.zeros(binding.denoise_graph_state_bytes(), dtype=torch.uint8, device=self.device)
        self._graph_keep = getattr(self, "_graph_keep", []) + [state, kt, vtt, x]
        return binding.denoise_graph_create(self.cfg, self.mw, self.cache, x, kt, vtt, list(stream_ids), n_frames,
                                            self.workspace(B, L), state)

    def cache_logical(self, layer, stream):
        """Host copies of one cache in token-row form: K, V float32 [S+W, C] and ids int64 [S+W]."""
        kp, vp, ip, cap = binding.kv_cache_device_ptrs(self.cache, layer, stream)
        base = self.cache_storage.data_ptr()
        H, D = self.wl.H, self.wl.D
        n = H * cap * D * 2
        kraw = self.cache_storage[kp - base:kp - base + n].view(torch.bfloat16).view(H, cap, D)
        vraw = self.cache_storage[vp - base:vp - base + n].view(torch.bfloat16).view(H, D, cap)
        ids = self.cache_storage[ip - base:ip - base + cap * 8].view(torch.int64)
        nslot = self.S + self.W
        K = kraw.permute(1, 0, 2).reshape(cap, H * D)[:nslot].float().cpu().numpy()
        vraw = vraw[:, :, binding.vt_columns(cap).to(vraw.device)]          # column order -> slot order
        V = vraw.permute(2, 0, 1).reshape(cap, H * D)[:nslot].float().cpu().numpy()
        return K, V, ids[:nslot].cpu().numpy()

    def state(self, layer, stream):
        return binding.kv_cache_state(self.cache, layer, stream)

    def slot_map(self, layer, stream):
        return np.asarray(binding.kv_cache_slot_map(self.cache, layer, stream, self.S + self.W), dtype=np.int64)

    def close(self):
        binding.kv_cache_destroy(self.cache)
