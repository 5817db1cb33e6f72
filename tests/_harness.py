"""Shared set-up for GPU parity tests: one seeded head, the oracle's index, the same index imported on the GPU."""
from __future__ import annotations

import sys
import time

import numpy as np

import synth
from oracle import csv_oracle as O

from . import _parity as PAR


def log(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


class Case:
    def __init__(self, recipe: synth.Recipe, seed: int = synth.SEED, bias: bool = True, radius_slack: float = 2.0 ** -14,
                 labels=None, B_max=None, K_cap=None, want_W64: bool = True, W_bits=None, centroid_bf16: bool = False,
                 bias_table_m: int = 0, b=None, angular: bool = False):
        import torch
        import paper_2511_21702_amd as csv
        self.csv, self.torch = csv, torch
        self.r = recipe
        t0 = time.time()
        self.head = synth.make_head(recipe, seed=seed, threads=16)
        if W_bits is not None:                      # a hand-made matrix in place of the generated one
            self.head = dict(self.head, W_bits=np.ascontiguousarray(W_bits))
        self.b = (self.head["b"] if b is None else b) if bias else None
        self.labels = self.head["labels"] if labels is None else labels
        self.C = recipe.C if labels is None else int(np.max(labels)) + 1
        log(f"[{recipe.name}] head V={recipe.V} d={recipe.d} C={self.C} generated in {time.time() - t0:.1f}s")
        t0 = time.time()
        if angular:
            self.oidx = O.build_index_angular(self.head["W_bits"], self.b, self.labels, self.C, slack=radius_slack)
        else:
            self.oidx = O.build_index(self.head["W_bits"], self.b, self.labels, self.C, radius_slack=radius_slack,
                                      centroid_bf16=centroid_bf16, bias_table_m=bias_table_m)
        log(f"[{recipe.name}] oracle index in {time.time() - t0:.1f}s")
        self.W64 = O.bf16_to_f64(self.head["W_bits"]) if want_W64 else None
        self.dW = csv.bits_to_device(self.head["W_bits"])
        self.db = None if self.b is None else torch.from_numpy(self.b).cuda()
        self.gidx = csv.csv_index_from_arrays(self.dW, self.db, self.oidx.mu, self.oidx.R, self.oidx.bmax,
                                              self.oidx.n.astype(np.int32), self.oidx.perm.astype(np.int32),
                                              centroid_bf16=centroid_bf16)
        if self.oidx.bias_table is not None:
            self.gidx.set_bias_table(self.oidx.bias_table)
        if self.oidx.ang is not None:
            self.gidx.set_angular(self.oidx.ang)
        self.ws = csv.CsvWorkspace(self.gidx, B_max or recipe.B, K_cap if K_cap is not None else recipe.K_max_rows)
        torch.cuda.synchronize()

    def hidden(self, steps=None, seed=synth.SEED):
        return synth.make_hidden(self.r, self.head["centers"], steps=steps, seed=seed)

    def run_steps(self, h_bits: np.ndarray, k: int, eps: float, K_max: int, combine: int, tag: str, tally=None,
                  step_ids=None, max_rounds: int = 2, delta_clusters: int = 0, relax: bool = False) -> PAR.Tally:
        """h_bits [steps,B,d].  Runs every step on the GPU; compares the steps in step_ids (default all) with the oracle."""
        csv, torch = self.csv, self.torch
        steps, B, d = h_bits.shape
        t = tally or PAR.Tally()
        dh = csv.bits_to_device(h_bits)
        buf = csv.make_step_buffers(self.gidx, B, k, eps, K_max, combine, want_sel=True, max_rounds=max_rounds,
                                    delta_clusters=delta_clusters, relax=relax)
        step_ids = list(range(steps)) if step_ids is None else list(step_ids)
        outs = []
        for s in step_ids:
            csv.csv_decode_step(self.ws, self.gidx, dh[s], buf)
            torch.cuda.synchronize()
            outs.append(PAR.gpu_step_to_numpy(buf))
        # oracle logits for several steps per matrix product (same values as step by step)
        group = max(1, 256 // B)
        for g0 in range(0, len(step_ids), group):
            ids = step_ids[g0:g0 + group]
            h64 = O.bf16_to_f64(h_bits[ids].reshape(-1, d))
            Lall = O.full_logits(self.W64, self.b, h64).reshape(len(ids), B, -1)
            for j, s in enumerate(ids):
                orc = O.decode_step(self.W64, self.b, self.oidx, h_bits[s], k, eps, K_max, combine, logits=Lall[j],
                                    max_rounds=max_rounds, delta_clusters=delta_clusters, relax=relax)
                PAR.compare_step(f"{tag} step={s}", t, orc, outs[g0 + j], Lall[j], self.oidx, k, eps, K_max, combine)
            log(f"[{tag}] compared steps {ids[0]}..{ids[-1]}: {t.summary()}")
        return t

    def close(self):
        self.ws.free()
        self.gidx.free()
