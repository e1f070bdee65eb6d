"""Host loop of a block-wise DepCap decode over a batch of independent sequences.

All arithmetic happens in libdlm (dlm_step, block_boundary, select_parallel); this file only
decides which pass each sequence needs next, packs the sequences of one iteration into one
launch of each entry point, and reads back two small integer arrays per iteration (the next
block lengths and the number of tokens written), because the shapes of the next launch depend
on them.

Pass schedule per sequence (Sec. 3 "Block-wise decoding", Sec. 4.2; Eq. 2 for the token write):
  prefill    span = prompt + look-ahead masks; the prompt joins the KV cache; the look-ahead logits
             are retained as p^prev; the first block has L = L_min (cold start)
  in-block   span = the current block against the cache; CAP-Decoding on its masked rows
  boundary   once a block is mask-free: span = block + look-ahead; the block joins the cache; the
             first min(L_max, remaining) look-ahead rows give I_k (KL to the retained p^prev) and
             H_k; block_boundary gives the next L; the look-ahead rows are retained as the new
             p^prev and double as the next block's first denoising step
"""
import numpy as np
import torch

from . import api


class Decoder:
    def __init__(self, model, batch, prompt_len, gen_len, prm, device, max_rows=None):
        """prm: dict(l_min, l_max, lam, smooth_radius, norm_mode, rule, tau_low, tau_high, gamma, mode[, fixed_block]).

        fixed_block = B > 0: every block has min(B, remaining) positions instead of the DepGA-Block length (the fixed block
        sizes of the comparison methods of Sec. 5.1); the boundary pass then compares and retains nothing.
        dual_cache = 1: in-block passes also attend to the look-ahead positions after the block, with the keys and values the
        last prefill / boundary pass left in the cache for them (the suffix half of a dual cache, Sec. 5.2, Q2)."""
        self.model, self.cfg, self.prm, self.device = model, model.cfg, dict(prm), device
        self.B, self.P, self.N = batch, prompt_len, gen_len
        self.T = prompt_len + gen_len
        lmax = prm["l_max"]
        self.fixed = int(prm.get("fixed_block", 0))
        self.dual = bool(prm.get("dual_cache", 0))
        self.look = min(2 * lmax, gen_len)
        steady = batch * (lmax + self.look)
        self.max_rows = max_rows or max(prompt_len + self.look, steady)
        self.state = api.State(model, batch, self.T, self.max_rows, self.look)
        self.out = api.StepOutputs(self.max_rows, self.cfg["vocab"], model.torch_dtype, device)
        self.tokens = torch.empty((batch, self.T), dtype=torch.int32, device=device)
        self.sel = torch.zeros(self.max_rows, dtype=torch.uint8, device=device)
        self.nsel = torch.zeros(batch, dtype=torch.int32, device=device)
        self.L_dev = torch.zeros(batch, dtype=torch.int32, device=device)
        self.time_steps = False  # bracket every dlm_step launch with events on the launch stream (measurement only)

    def load(self, prompts):
        """prompts: int array [B, P]; generation slots are filled with the mask id."""
        t = np.full((self.B, self.T), self.cfg["mask_id"], dtype=np.int32)
        t[:, : self.P] = prompts
        self.tokens.copy_(torch.from_numpy(t))
        for b in range(self.B):
            self.state.reset(b)
        # per sequence: frontier F, block length L, masks left in the block, phase
        self.F = [self.P] * self.B
        self.L = [0] * self.B
        self.left = [0] * self.B
        self.phase = ["prefill"] * self.B
        self.look_end = [0] * self.B  # end of the positions the sequence's last prefill / boundary pass covered
        self.nfe, self.blocks, self.steps = [0] * self.B, [[] for _ in range(self.B)], [[] for _ in range(self.B)]
        self.launches = 0
        self.rows_log = []  # rows of every dlm_step launch
        self.pass_log = []  # per launch: (rows of each packed sequence, cached prefix length of each)
        self.kl_rows = 0    # rows compared with their retained distribution (Eq. 3), all launches together
        self.stat_log = []  # per launch: (rows, rows compared with or retained as a previous-step distribution)
        self.step_events = []  # (rows, start, end) events around every dlm_step launch when time_steps is set
        self.kind_counts = dict(prefill=0, inblock=0, boundary=0)  # passes of each kind, all sequences together

    def _plan(self, b):
        """(span_start, rows, commit, kl_first, kl_count, save_first, save_count) of sequence b's next pass."""
        END, lmax = self.T, self.prm["l_max"]
        if self.phase[b] == "prefill":
            return 0, self.P + self.look, self.P, 0, 0, self.P, (0 if self.fixed else self.look)
        F, L = self.F[b], self.L[b]
        if self.phase[b] == "inblock":
            return F, L, 0, 0, 0, 0, 0
        R = END - (F + L)
        Lk, W = min(2 * lmax, R), min(lmax, R)
        if self.fixed:
            return F, L + Lk, L, L, 0, L, 0
        return F, L + Lk, L, L, W, L, Lk

    def iterate(self, trace=None):
        """One iteration: every unfinished sequence gets its next pass and its next selection."""
        prm, lmax = self.prm, self.prm["l_max"]
        todo = [b for b in range(self.B) if self.phase[b] != "done"]
        while todo:
            # pack as many sequences as fit into max_rows
            group, rows, plans = [], 0, {}
            while todo:
                p = self._plan(todo[0])
                if group and rows + p[1] > self.max_rows:
                    break
                b = todo.pop(0)
                group.append(b)
                plans[b] = p
                rows += p[1]
            self._launch(group, plans, trace)

    def _launch(self, group, plans, trace):
        prm, lmax, out = self.prm, self.prm["l_max"], self.out
        row_off = [0]
        for b in group:
            row_off.append(row_off[-1] + plans[b][1])
        col = lambda i: [plans[b][i] for b in group]
        if trace is not None:  # the tokens this pass reads, before the selection below rewrites some of them
            self._fed = [self.tokens[b, plans[b][0]: plans[b][0] + plans[b][1]].cpu().numpy() for b in group]
        if self.time_steps:
            ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            ev[0].record()
        suffix = [self.look_end[b] - (plans[b][0] + plans[b][1]) if (self.dual and self.phase[b] == "inblock") else 0 for b in group]
        api.dlm_step(self.state, self.tokens, out, row_off, col(0), col(2), [b * self.T + plans[b][0] for b in group], slot=group,
                     kl_first=col(3), kl_count=col(4), save_first=col(5), save_count=col(6), suffix_len=suffix)
        for b in group:
            if self.phase[b] != "inblock":
                self.look_end[b] = plans[b][0] + plans[b][1]
        if self.time_steps:
            ev[1].record()
            self.step_events.append((row_off[-1], ev[0], ev[1]))
        self.launches += 1
        self.rows_log.append(row_off[-1])
        self.pass_log.append(([plans[b][1] for b in group], [plans[b][0] for b in group]))
        self.kl_rows += sum(plans[b][4] for b in group)
        self.stat_log.append((row_off[-1], sum(plans[b][4] + plans[b][6] for b in group)))
        for b in group:
            self.nfe[b] += 1
            self.kind_counts[self.phase[b]] += 1
        # block-boundary decisions for the sequences that just finished a block (or the prompt)
        bnd = [i for i, b in enumerate(group) if self.phase[b] != "inblock"]
        if bnd and self.fixed:
            for i in bnd:
                b = group[i]
                self.F[b] += self.L[b]
                self.L[b] = self.left[b] = min(self.fixed, self.T - self.F[b])
                self.blocks[b].append(self.L[b])
        elif bnd:
            starts, lens, cold = [], [], []
            for i in bnd:
                b = group[i]
                sp, rws, commit, klf, klc, _, _ = plans[b]
                if self.phase[b] == "prefill":
                    starts.append(row_off[i] + self.P)
                    lens.append(min(lmax, self.N))
                    cold.append(1)
                else:
                    starts.append(row_off[i] + klf)
                    lens.append(klc)
                    cold.append(0)
            api.block_boundary(out.kl, out.entropy, starts, lens, self.L_dev, prm["lam"], prm["l_min"], prm["smooth_radius"],
                               prm["norm_mode"], prm["rule"], cold=cold)
            Ls = self.L_dev[: len(bnd)].cpu().numpy()
            for j, i in enumerate(bnd):
                b = group[i]
                if trace is not None:
                    trace.append(dict(op="boundary", seq=b, F=self.F[b] + self.L[b], W=lens[j], L=int(Ls[j]), cold=bool(cold[j]),
                                      kl=out.kl[starts[j]: starts[j] + lens[j]].cpu().numpy(),
                                      entropy=out.entropy[starts[j]: starts[j] + lens[j]].cpu().numpy()))
                self.F[b] += self.L[b]
                self.L[b] = self.left[b] = int(Ls[j])
                self.blocks[b].append(self.L[b])
        # CAP-Decoding on the current block of every sequence of the group
        row_start = []
        for i, b in enumerate(group):
            first = 0 if self.phase[b] == "inblock" else plans[b][2]  # the block follows the committed rows
            row_start.append(row_off[i] + first)
        blen = [self.L[b] for b in group]
        api.select_parallel(out.logits, out.lse, out.conf, out.argmax, self.tokens, row_start, [b * self.T + self.F[b] for b in group],
                            blen, self.cfg["mask_id"], prm["tau_low"], prm["tau_high"], prm["gamma"], prm.get("mode", 0), self.sel,
                            self.nsel, apply_tokens=True)
        ns = self.nsel[: len(group)].cpu().numpy()
        if trace is not None:
            for i, b in enumerate(group):
                sp, rws = plans[b][0], plans[b][1]
                trace.append(dict(op="pass", seq=b, kind=self.phase[b] if self.phase[b] != "prefill" else "prefill", span_start=sp,
                                  rows=rws, commit_len=plans[b][2], tokens=self._fed[i],
                                  logits=out.logits[row_off[i]: row_off[i] + rws].cpu()))
                trace.append(dict(op="select", seq=b, F=self.F[b], L=self.L[b],
                                  selected=self.sel[row_start[i]: row_start[i] + blen[i]].cpu().numpy().astype(bool)))
        for i, b in enumerate(group):
            self.steps[b].append(int(ns[i]))
            self.left[b] -= int(ns[i])
            if self.left[b] > 0:
                self.phase[b] = "inblock"
            elif self.F[b] + self.L[b] >= self.T:
                self.phase[b] = "done"
            else:
                self.phase[b] = "boundary"

    def run(self, prompts, trace=None):
        self.load(prompts)
        while any(p != "done" for p in self.phase):
            self.iterate(trace)
        torch.cuda.synchronize()
        return dict(tokens=self.tokens.cpu().numpy().astype(np.int64), nfe=list(self.nfe), blocks=self.blocks, steps=self.steps,
                    launches=self.launches)

    def close(self):
        self.state.close()
