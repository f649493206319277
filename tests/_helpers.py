"""Shared plumbing for the GPU parity tests: builds the same layer on both
sides from one set of seeded input bytes, and the error metric."""
import numpy as np
import torch

from oracle import skv_oracle as O
from paper_2601_21686_amd import binding as B
from paper_2601_21686_amd import synth

TOL = 2e-3      # max relative error of an output vector (fp32 accumulate, bf16 storage)


def vec_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over output vectors of ||got - want||_inf / ||want||_inf."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    num = np.max(np.abs(got - want), axis=1)
    den = np.max(np.abs(want), axis=1)
    return float(np.max(num / den))


def elem_rel_err(got: np.ndarray, want: np.ndarray, floor: float = 1e-3) -> float:
    """max over elements of |got - want| / max(|want|, floor * ||want||_inf of the element's vector): the plain
    element-wise relative error, with an absolute floor so that entries near zero do not decide it.  Logged
    beside vec_rel_err; the tolerance is stated for vec_rel_err."""
    got = np.asarray(got, np.float64).reshape(-1, got.shape[-1])
    want = np.asarray(want, np.float64).reshape(-1, want.shape[-1])
    den = np.maximum(np.abs(want), floor * np.max(np.abs(want), axis=1, keepdims=True))
    return float(np.max(np.abs(got - want) / den))


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in units of bf16 steps between two arrays of bit patterns."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7fff), x & 0x7fff)
    return np.abs(key(a_bits) - key(b_bits))


class Pair:
    """A GPU layer (binding.Layer) and an oracle layer holding the same bases."""

    def __init__(self, seed, batch, hq, hkv, r_k, r_v, capacity, shared_k=False, shared_v=False,
                 device="cuda", fill_bits=None, oracle=True):
        self.batch, self.hq, self.hkv, self.r_k, self.r_v, self.capacity = batch, hq, hkv, r_k, r_v, capacity
        self.device = device
        _, pk = synth.orthonormal_bases(synth.stable_seed(seed, "pk"), 1 if shared_k else hkv, 128, r_k)
        _, pv = synth.orthonormal_bases(synth.stable_seed(seed, "pv"), 1 if shared_v else hkv, 128, r_v)
        self.pk_bits = synth.torch_bf16_to_bits(pk)
        self.pv_bits = synth.torch_bf16_to_bits(pv)
        kc = vc = None
        if fill_bits is not None:
            kc = torch.full((batch, hkv, capacity, r_k), fill_bits, dtype=torch.int16, device=device).view(torch.bfloat16)
            vc = torch.full((batch, hkv, capacity, r_v), fill_bits, dtype=torch.int16, device=device).view(torch.bfloat16)
        self.gpu = B.Layer(batch, hq, hkv, pk.to(device), pv.to(device), capacity, kc, vc)
        self.scales_k = synth.channel_scales(synth.stable_seed(seed, "sk"), hkv, 128)
        self.scales_v = synth.channel_scales(synth.stable_seed(seed, "sv"), hkv, 128)
        self.ora = None
        if oracle:
            self.ora = O.new_layer(batch, hq, hkv, 128, O.bf16_bits_to_f64(self.pk_bits),
                                   O.bf16_bits_to_f64(self.pv_bits), capacity, store="bf16")

    def raw_kv(self, seed, T, device=None):
        device = device or self.device
        k = synth.kv_activations(synth.stable_seed(seed, "k"), self.batch, T, self.hkv, 128, self.scales_k, device)
        v = synth.kv_activations(synth.stable_seed(seed, "v"), self.batch, T, self.hkv, 128, self.scales_v, device)
        return k, v

    def oracle_append(self, k, v, cur_len):
        O.project_append(self.ora, O.bf16_bits_to_f64(synth.torch_bf16_to_bits(k)),
                         O.bf16_bits_to_f64(synth.torch_bf16_to_bits(v)), cur_len)

    def upload_oracle_cache(self, n):
        """Copies rows [0, n) of the oracle's cache (its own bf16 bits) to the GPU layer."""
        kb = O.f64_to_bf16_bits(self.ora.k_cache[:, :, :n])
        vb = O.f64_to_bf16_bits(self.ora.v_cache[:, :, :n])
        self.gpu.k_cache[:, :, :n] = synth.bits_to_torch_bf16(kb, self.device)
        self.gpu.v_cache[:, :, :n] = synth.bits_to_torch_bf16(vb, self.device)

    def queries(self, seed):
        return synth.queries(synth.stable_seed(seed, "q"), self.batch, self.hq, 128, self.device)

    def oracle_decode(self, q, n_ctx, scale=None, heads=None):
        return O.decode_attention(self.ora, O.bf16_bits_to_f64(synth.torch_bf16_to_bits(q)), n_ctx, scale, heads)

    def gpu_decode(self, q, n_ctx, scale=0.0):
        out = torch.empty((self.batch, self.hq, 128), dtype=torch.float32, device=self.device)
        B.skv_decode_attention(self.gpu, q, out, n_ctx, scale)
        torch.cuda.synchronize()
        return out.cpu().numpy()
