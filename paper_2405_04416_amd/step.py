"""One forward + backward pass of the DistGrid hot path on one GPU: call sequencing only.

`TrainStep` owns the device buffers and issues the library calls in the order of the paper's
training procedure (Sec. 4.4.2, Fig. 2): ray/box segments -> distribution to the resident
sub-models -> per sub-model sampling, encode, MLPs, local compositing -> merge -> loss seeds ->
merge backward (Eq. 7-8) -> per sub-model compositing / MLP / encode backward.  Every arithmetic
step happens inside libdistgrid; this file allocates, slices and calls.
"""
import contextlib

import torch

from . import binding as B


def split_appearance_columns(w, desc):
    """Packed MLP weights (or their gradient; numpy) with ONE wide first colour layer [n_hidden_c, n_geo + n_dir + n_app]
    -> the library's packing: the matrices without the appearance columns first, those columns
    Wapp [n_hidden_c, n_app] last.  Pure re-arrangement."""
    import numpy as np
    if not desc.n_app:
        return w
    pos = desc.n_hidden_d * desc.n_feat + desc.n_geo * desc.n_hidden_d
    no, ni = desc.n_hidden_c, desc.n_geo + desc.n_dir + desc.n_app
    Wc1 = np.asarray(w[pos:pos + no * ni]).reshape(no, ni)
    return np.concatenate([w[:pos], Wc1[:, :ni - desc.n_app].ravel(), w[pos + no * ni:], Wc1[:, ni - desc.n_app:].ravel()])


class SubModel:
    """Parameters and gradient buffers of one partition's sub-NeRF (hash table + MLP weights)."""

    def __init__(self, grid_desc, mlp_desc, table, weights):
        self.grid, self.mlp = grid_desc, mlp_desc
        self.table, self.weights = table, weights
        self.dtable = torch.zeros_like(table)
        self.dW = torch.zeros(weights.numel(), dtype=torch.float32, device=weights.device)
        self.opt = None     # optimiser state, allocated by the first optimiser step

    def optimiser_state(self):
        """Adam moments of the table and of the weights, and the fp32 master copy of the fp16 weights."""
        if self.opt is None:
            self.opt = {"table_m": torch.zeros_like(self.table), "table_v": torch.zeros_like(self.table),
                        "w_master": self.weights.float().reshape(-1).contiguous(), "w_m": torch.zeros_like(self.dW),
                        "w_v": torch.zeros_like(self.dW)}
        return self.opt


class Occupancy:
    """Occupancy grid of one sub-model (Sec. 3.2, Sec. 5.1): geometry, per-cell densities, bit field, marching step."""

    def __init__(self, desc, density, bits, dt, max_steps):
        self.desc, self.density, self.bits, self.dt, self.max_steps = desc, density, bits, float(dt), int(max_steps)
        self.n_set = torch.zeros(1, dtype=torch.int32, device=density.device)


class TrainStep:
    def __init__(self, parts, models, resident, R, S, k_max, sh_degree, loss_scale=65536.0, lambda1=0.0, seed=0,
                 device="cuda:0", max_segments=None, binned_backward=True, encode_ws_cap=48 << 30, holes=None,
                 occupancy=None, max_samples=None, appearance=None, foreign_prefilled=False):
        """parts: [P,6] float tensor (device); models: {partition index: SubModel}; resident: partition indices served;
        max_segments: room for the segments of the RESIDENT partitions (default R * k_max);
        foreign_prefilled: the caller keeps the partial slots Ck / Tk of segments in non-resident partitions filled (in a
        deployment the exchange of Fig. 2 step 5 writes them); otherwise a step with non-resident partitions needs a
        `foreign` callable or it raises -- such slots are never silently read as whatever the buffers hold;
        holes: None or [P,6] (device): the box subtracted from each partition (coarse level of the cascade, Sec. 4.2.2);
        occupancy: None (S stratified samples per segment) or {partition index: Occupancy}: occupancy-guided sampling
        (Sec. 3.2, Sec. 5.1), at most max_samples samples per step over all resident partitions (S is then unused);
        appearance: None or (table [n_images, n_app] fp16, image_of_ray [R] int32), both on the device: per-image
        appearance vectors as further colour-net inputs (Sec. 4.4.3; the sub-models' MLP descriptors carry n_app)."""
        self.dev = torch.device(device)
        self.parts, self.models, self.resident, self.holes = parts, models, list(resident), holes
        self.parts_host = parts.cpu().tolist()
        self.P, self.R, self.S, self.k_max, self.deg = parts.shape[0], R, S, k_max, sh_degree
        self.loss_scale, self.lambda1, self.seed = float(loss_scale), float(lambda1), seed
        i32, f32, f16 = torch.int32, torch.float32, torch.float16
        z = lambda *shape, dt=f32: torch.zeros(*shape, dtype=dt, device=self.dev)
        cap = R * k_max if max_segments is None else max_segments
        self.cap = cap
        self.seg_count, self.seg_t, self.seg_part = z(R, dt=i32), z(R, k_max, 2), z(R, k_max, dt=i32)
        self.part_offset, self.status = z(self.P + 1, dt=i32), z(1, dt=i32)
        self.seg_ray, self.seg_slot = z(R * k_max, dt=i32), z(R * k_max, dt=i32)
        self.ws_seg = z(max(B.dg_segments_workspace_bytes(R, self.P) // 4, 1), dt=i32)
        self.occ = occupancy
        n = cap * S if occupancy is None else int(max_samples)
        self.max_samples = n
        any_model = next(iter(models.values()))
        self.n_feat = any_model.grid.n_levels * any_model.grid.n_features
        self.u, self.delta = z(n, 3), z(n)
        self.dir_enc = z(cap if occupancy is None else n, sh_degree * sh_degree, dt=f16)
        if occupancy is not None:
            self.first = z(R * k_max + self.P + 1, dt=i32)   # per partition: n_seg + 1 sample offsets, at [b + p, e + p]
            self.t, self.sample_ray = z(n), z(n, dt=i32)
            self.ws_march = z(B.dg_march_workspace_bytes(cap) // 4, dt=i32)
            self.samples = {}                               # partition -> (first sample, number of samples) of this step
        self.appearance = appearance
        self.app_rows = None if appearance is None else z(self.dir_enc.shape[0], appearance[0].shape[1], dt=f16)
        self.feat = z(n, self.n_feat, dt=f16)
        self.sigma, self.rgb = z(n), z(n, 3)
        self.dsigma, self.drgb = z(n), z(n, 3)
        self.dfeat = z(n, self.n_feat)
        self.Ck, self.Tk = z(R, k_max, 3), z(R, k_max)
        self.gCk, self.gTk = z(R, k_max, 3), z(R, k_max)
        self.C, self.T, self.gC, self.gT = z(R, 3), z(R), z(R, 3), z(R)
        self.loss = z(1)
        self.ws_mlp = z(B.dg_mlp_bwd_app_workspace_bytes(any_model.mlp, n, S if occupancy is None else 1) // 4 + 64)
        # workspace of the binned table-gradient pass, capped (the call batches itself when it is smaller than ideal)
        want = max(B.dg_hashgrid_encode_bwd_workspace_bytes(mm.grid, n) for mm in models.values())
        self.ws_enc = torch.zeros(min(want, encode_ws_cap) // 4 + 64, dtype=f32, device=self.dev) if binned_backward else None
        self.foreign_prefilled = bool(foreign_prefilled)
        # The queue sizes of the binned table-gradient pass depend on the sample coordinates alone: for the sub-model whose
        # backward pass comes first they are counted on a second stream as soon as its samples exist, beside the forward
        # pass (which waits for memory and leaves the arithmetic units idle), together with the clearing of its gradient
        # buffers.  One workspace serves all sub-models, so only one count can be ahead.  (Counts ahead for every sub-model,
        # each in a workspace of its own, were measured on four and eight resident sub-models: no gain, 32.5 against 32.3 ms
        # and 40.0 against 40.0 ms per step.)
        self.side = torch.cuda.Stream(device=self.dev) if binned_backward and occupancy is None else None
        self.counted = None     # (partition, samples, event) of a count that is ahead
        self.offsets = None
        self.local = {}         # resident partition -> index of its first segment among the resident segments (sample buffers)
        self.t_fixed = None
        self.timings = None     # set to {} to collect (start, end) event pairs per entry point

    @contextlib.contextmanager
    def _timed(self, name):
        """Brackets one library call with events on the stream it is launched on (the current stream)."""
        if self.timings is None:
            yield
            return
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        yield
        b.record()
        self.timings.setdefault(name, []).append((a, b))

    def timing_summary(self):
        """{entry point: (calls, total ms)} from the collected events; synchronises."""
        torch.cuda.synchronize()
        return {k: (len(v), sum(a.elapsed_time(b) for a, b in v)) for k, v in (self.timings or {}).items()}

    # -- forward ---------------------------------------------------------------------------
    def segments(self, o, d, t_min=0.0):
        self.status.zero_()
        with self._timed("dg_ray_aabb_segments"):
            B.dg_ray_aabb_segments(o, d, self.parts, t_min, self.k_max, self.seg_count, self.seg_t, self.seg_part,
                                   self.status, self.part_offset, self.seg_ray, self.seg_slot, self.ws_seg, holes=self.holes)
        self.offsets = self.part_offset.cpu().tolist()      # P+1 integers: how many segments each sub-model got
        # the sample buffers hold the segments of the resident partitions only, back to back in the order of `resident`
        run = 0
        for p in self.resident:
            self.local[p] = run
            run += self.offsets[p + 1] - self.offsets[p]
        if run > self.cap:
            raise B.DistGridError("segment capacity %d exceeded (%d)" % (self.cap, run))

    def _slices(self, p):
        """Segment range [b, e) of partition p in seg_ray / seg_slot, and the range of its samples in the sample buffers."""
        b, e = self.offsets[p], self.offsets[p + 1]
        first = self.local[p]
        return b, e, slice(first * self.S, (first + e - b) * self.S)

    def _rows(self, p):
        """Rows of partition p in the per-segment tables (direction encoding, appearance rows)."""
        first = self.local[p]
        return slice(first, first + self.offsets[p + 1] - self.offsets[p])

    def forward(self, o, d, Cgt, jitter=None, foreign=None):
        """foreign: optional callable(self) that fills partials of non-resident partitions into Ck/Tk."""
        if foreign is None and not self.foreign_prefilled and len(self.resident) < self.P:
            raise B.DistGridError("partitions %s are not resident: pass `foreign` to fill their partials, or construct with "
                                  "foreign_prefilled=True" % sorted(set(range(self.P)) - set(self.resident)))
        self._partials(o, d, jitter, training=True)
        if foreign is not None:
            foreign(self)
        with self._timed("dg_merge_segments"):
            B.dg_merge_segments(self.Ck, self.Tk, self.seg_count, self.R, self.k_max, self.C, self.T)
        self.loss.zero_()
        with self._timed("dg_loss_seed"):
            B.dg_loss_seed(self.C, self.T, Cgt, self.R, self.lambda1, self.gC, self.gT, self.loss)

    def render(self, o, d, jitter=None, fused=None):
        """Evaluation rendering (Sec. 4.4.2): forward only, every sub-model renders its segments and the partial
        results are merged into the final colour, depth and transmittance.  Returns (C [R,3], D [R], T [R]).
        fused: None = use the fused networks + rendering kernel where it applies; False = the separate entry points."""
        if self.occ is None and self.t_fixed is None:
            self.t_fixed = torch.zeros_like(self.delta)          # sample distances, only evaluation needs them
        Dk = torch.zeros(self.R, self.k_max, device=self.dev)
        D = torch.zeros(self.R, device=self.dev)
        # networks and local rendering in one kernel where the library has one (fixed S <= 64, the 32-64-16 / 64-64-3 nets)
        mlp = next(iter(self.models.values())).mlp
        fused = fused if fused is not None else (self.occ is None and self.S <= 64 and (mlp.n_feat, mlp.n_hidden_d, mlp.n_layers_c) == (32, 64, 2))
        self._partials(o, d, jitter, want_t=True, fused_depth=Dk if fused else None)
        B.dg_merge_segments(self.Ck, self.Tk, self.seg_count, self.R, self.k_max, self.C, self.T)
        if self.occ is not None:
            return self.C, self.depth(), self.T
        for p in () if fused else self.resident:
            b, e, sl = self._slices(p)
            if e > b:
                B.dg_composite_segment_depth(self.sigma[sl], self.delta[sl], self.t_fixed[sl], e - b, self.S, self.seg_ray[b:e],
                                             self.seg_slot[b:e], self.k_max, Dk)
        B.dg_merge_depth(Dk, self.Tk, self.seg_count, self.R, self.k_max, D)
        return self.C, D, self.T

    def _count_ahead(self, p, sl, N):
        """Starts the count sweep of sub-model p's table-gradient pass (and clears its gradient buffers) on the second
        stream, behind the work already queued on this one; the backward pass picks it up."""
        m = self.models[p]
        if B.dg_hashgrid_encode_bwd_workspace_bytes(m.grid, N) > self.ws_enc.numel() * self.ws_enc.element_size():
            return                                  # the workspace would batch: counted with each batch, as usual
        here = torch.cuda.Event()
        here.record()
        go = torch.cuda.Event()
        with torch.cuda.stream(self.side):
            self.side.wait_event(here)
            go.record()
            B.dg_hashgrid_encode_bwd_count(m.grid, self.u[sl], N, self.ws_enc)
            m.dtable.zero_()
            m.dW.zero_()
            done = torch.cuda.Event()
            done.record()
        # this stream goes on once the second one has got that far: the count sweep's few workgroups are then handed out
        # before the forward gather's millions arrive and fill every wavefront slot of the chip
        torch.cuda.current_stream().wait_event(go)
        self.counted = (p, N, done)

    def _partials(self, o, d, jitter=None, want_t=False, fused_depth=None, training=False):
        """Segments, and per resident sub-model: samples, encode, MLPs, local compositing into the partial slots.
        fused_depth: None, or Dk [R,k_max]: networks, compositing and depth in one call (evaluation rendering)."""
        self.counted = None
        S = self.S
        self.segments(o, d)
        # the sub-model whose backward pass runs first: only its counts may wait in the workspace that all share
        first = next((p for p in self.resident if self.offsets[p + 1] > self.offsets[p]), None)
        if self.occ is not None:
            self._forward_marched(o, d)
        for p in self.resident if self.occ is None else ():
            b, e, sl = self._slices(p)
            n_seg = e - b
            if n_seg == 0:
                continue
            m = self.models[p]
            N = n_seg * S
            jit = None if jitter is None else jitter[sl]
            with self._timed("dg_sample_segments"):
                B.dg_sample_segments(o, d, self.seg_t, self.seg_ray[b:e], self.seg_slot[b:e], n_seg, self.k_max,
                                     self.parts_host[p], S, self.seed, jit, self.u[sl], self.delta[sl],
                                     self.t_fixed[sl] if want_t else None)
            rows = self._rows(p)
            if training and self.side is not None and p == first:
                self._count_ahead(p, sl, N)
            with self._timed("dg_dir_encode"):
                B.dg_dir_encode(d, self.seg_ray[b:e], n_seg, self.deg, self.dir_enc[rows])
            with self._timed("dg_hashgrid_encode_fwd"):
                B.dg_hashgrid_encode_fwd(m.grid, m.table, self.u[sl], N, self.feat[sl])
            app = self._appearance_rows(self.seg_ray[b:e], n_seg, rows)
            if fused_depth is not None:
                with self._timed("dg_mlp_composite_fwd"):
                    B.dg_mlp_composite_fwd(m.mlp, m.weights, self.feat[sl], self.dir_enc[rows], app, S, n_seg, self.delta[sl],
                                           self.t_fixed[sl], self.seg_ray[b:e], self.seg_slot[b:e], self.k_max, self.Ck, self.Tk,
                                           fused_depth)
                continue
            with self._timed("dg_mlp_fwd"):
                B.dg_mlp_fwd_app(m.mlp, m.weights, self.feat[sl], self.dir_enc[rows], app, S, N, self.sigma[sl], self.rgb[sl])
            with self._timed("dg_composite_segment_fwd"):
                B.dg_composite_segment_fwd(self.sigma[sl], self.rgb[sl], self.delta[sl], n_seg, S, self.seg_ray[b:e],
                                           self.seg_slot[b:e], self.k_max, self.Ck, self.Tk)

    def _appearance_rows(self, index, n, rows):
        """Gathers the appearance vector of each row's ray (rows as for the direction encoding); None without them."""
        if self.appearance is None:
            return None
        with self._timed("dg_appearance_rows"):
            B.dg_appearance_rows(self.appearance[0], self.appearance[1], index, n, self.app_rows[rows])
        return self.app_rows[rows]

    def _forward_marched(self, o, d):
        """Per sub-model forward with occupancy-guided sampling (Sec. 3.2, Sec. 5.1): segments of different lengths,
        one direction row per sample."""
        self.samples = {}
        s0 = 0
        for p in self.resident:
            b, e = self.offsets[p], self.offsets[p + 1]
            n_seg = e - b
            if n_seg == 0:
                continue
            m, q = self.models[p], self.occ[p]
            first = self.first[b + p:e + p + 1]
            ray, slot = self.seg_ray[b:e], self.seg_slot[b:e]
            room = self.max_samples - s0
            with self._timed("dg_march_segments"):
                B.dg_march_segments(o, d, self.seg_t, ray, slot, n_seg, self.k_max, self.parts_host[p], q.desc, q.bits, q.dt,
                                    q.max_steps, self.seed, room, first, self.u[s0:], self.delta[s0:], self.t[s0:],
                                    self.sample_ray[s0:], self.status, self.ws_march)
            N = int(first[n_seg].item())                    # the one number the host needs: how many samples were kept
            if N > room:
                raise B.DistGridError("sample capacity %d exceeded (%d more wanted by partition %d)" % (self.max_samples, N - room, p))
            sl = slice(s0, s0 + N)
            self.samples[p] = (s0, N)
            s0 += N
            if N:
                with self._timed("dg_dir_encode"):
                    B.dg_dir_encode(d, self.sample_ray[sl], N, self.deg, self.dir_enc[sl])
                with self._timed("dg_hashgrid_encode_fwd"):
                    B.dg_hashgrid_encode_fwd(m.grid, m.table, self.u[sl], N, self.feat[sl])
                app = self._appearance_rows(self.sample_ray[sl], N, sl)
                with self._timed("dg_mlp_fwd"):
                    B.dg_mlp_fwd_app(m.mlp, m.weights, self.feat[sl], self.dir_enc[sl], app, 1, N, self.sigma[sl], self.rgb[sl])
            with self._timed("dg_composite_ragged_fwd"):        # also writes C_k = 0, T_k = 1 for segments that saw nothing
                B.dg_composite_ragged_fwd(self.sigma[s0 - N:], self.rgb[s0 - N:], self.delta[s0 - N:], n_seg, first, ray, slot,
                                          self.k_max, self.Ck, self.Tk)

    def depth(self):
        """Depth channel of evaluation rendering (Sec. 4.4.2) for the samples of the last forward pass with
        occupancy-guided sampling; returns D [R]."""
        Dk = torch.zeros(self.R, self.k_max, device=self.dev)
        D = torch.zeros(self.R, device=self.dev)
        for p, (s0, N) in self.samples.items():
            b, e = self.offsets[p], self.offsets[p + 1]
            B.dg_composite_ragged_depth(self.sigma[s0:], self.delta[s0:], self.t[s0:], e - b, self.first[b + p:e + p + 1],
                                        self.seg_ray[b:e], self.seg_slot[b:e], self.k_max, Dk)
        B.dg_merge_depth(Dk, self.Tk, self.seg_count, self.R, self.k_max, D)
        return D

    def _backward_marched(self):
        for p in self.resident:
            m = self.models[p]
            with self._timed("zero_gradients"):
                m.dtable.zero_()
                m.dW.zero_()
            if p not in self.samples or self.samples[p][1] == 0:
                continue
            s0, N = self.samples[p]
            b, e = self.offsets[p], self.offsets[p + 1]
            sl = slice(s0, s0 + N)
            with self._timed("dg_composite_ragged_bwd"):
                B.dg_composite_ragged_bwd(self.sigma[s0:], self.rgb[s0:], self.delta[s0:], e - b, self.first[b + p:e + p + 1],
                                          self.seg_ray[b:e], self.seg_slot[b:e], self.k_max, self.gCk, self.gTk, self.dsigma[s0:],
                                          self.drgb[s0:])
            with self._timed("dg_mlp_bwd"):
                B.dg_mlp_bwd_app(m.mlp, m.weights, self.feat[sl], self.dir_enc[sl], None if self.app_rows is None else self.app_rows[sl],
                                 1, N, self.dsigma[sl], self.drgb[sl], self.loss_scale, self.dfeat[sl], m.dW, self.ws_mlp)
            with self._timed("dg_hashgrid_encode_bwd"):
                B.dg_hashgrid_encode_bwd(m.grid, self.u[sl], self.dfeat[sl], N, m.dtable, self.ws_enc)

    # -- occupancy refresh (Sec. 5.1; Instant-NGP App. E.2) -------------------------------------
    def refresh_occupancy(self, iteration, tries=32):
        """Decay, candidate cells, the field's density at a random point of each, maximum, new bits -- when the
        schedule asks for it at this iteration.  Candidates are produced in pieces that fit the sample buffers, which
        serve as scratch: call it between training steps, not between a forward and its backward pass."""
        update_now, warmup, decay, threshold = B.dg_occ_schedule(iteration)
        if not update_now:
            return False
        for p in self.resident:
            m, q = self.models[p], self.occ[p]
            n_cells = q.desc.n_cells
            with self._timed("dg_occ_decay"):
                B.dg_occ_decay(q.density, decay)
            M = n_cells if warmup else n_cells // 2
            n_uniform = 0 if warmup else M // 2
            piece = self.max_samples
            for i0 in range(0, M, piece):
                n = min(piece, M - i0)
                cell = self.sample_ray[:n]                      # the step's sample buffers serve as scratch
                with self._timed("dg_occ_candidates"):
                    B.dg_occ_candidates(q.desc, q.bits, n, n_uniform, warmup, self.seed, iteration, tries, cell, self.u[:n], i0=i0)
                with self._timed("dg_hashgrid_encode_fwd"):
                    B.dg_hashgrid_encode_fwd(m.grid, m.table, self.u[:n], n, self.feat[:n])
                self.dir_enc[:1].zero_()                        # the density does not depend on the direction: one zero row
                if self.app_rows is not None:
                    self.app_rows[:1].zero_()
                with self._timed("dg_mlp_fwd"):
                    B.dg_mlp_fwd_app(m.mlp, m.weights, self.feat[:n], self.dir_enc[:1], None if self.app_rows is None else self.app_rows[:1],
                                     max(n, 1), n, self.sigma[:n], self.rgb[:n])
                with self._timed("dg_occ_update"):
                    B.dg_occ_update(q.density, cell, self.sigma[:n], n)
            q.n_set.zero_()
            with self._timed("dg_occ_bits"):
                B.dg_occ_bits(q.density, threshold, q.bits, q.n_set)
        return True

    # -- backward --------------------------------------------------------------------------
    def backward(self):
        S = self.S
        with self._timed("dg_merge_segments_bwd"):
            B.dg_merge_segments_bwd(self.Ck, self.Tk, self.seg_count, self.R, self.k_max, self.gC, self.gT, self.gCk,
                                    self.gTk)
        if self.occ is not None:
            return self._backward_marched()
        for p in self.resident:
            b, e, sl = self._slices(p)
            n_seg = e - b
            m = self.models[p]
            ahead = self.counted is not None and self.counted[0] == p
            if ahead:
                torch.cuda.current_stream().wait_event(self.counted[2])     # queues counted, gradient buffers cleared
                self.counted = None
            else:
                with self._timed("zero_gradients"):
                    m.dtable.zero_()
                    m.dW.zero_()
            if n_seg == 0:
                continue
            N = n_seg * S
            with self._timed("dg_composite_segment_bwd"):
                B.dg_composite_segment_bwd(self.sigma[sl], self.rgb[sl], self.delta[sl], n_seg, S, self.seg_ray[b:e],
                                           self.seg_slot[b:e], self.k_max, self.gCk, self.gTk, self.dsigma[sl], self.drgb[sl])
            rows = self._rows(p)
            with self._timed("dg_mlp_bwd"):
                B.dg_mlp_bwd_app(m.mlp, m.weights, self.feat[sl], self.dir_enc[rows], None if self.app_rows is None else self.app_rows[rows],
                                 S, N, self.dsigma[sl], self.drgb[sl], self.loss_scale, self.dfeat[sl], m.dW, self.ws_mlp)
            with self._timed("dg_hashgrid_encode_bwd"):
                if ahead:
                    B.dg_hashgrid_encode_bwd_counted(m.grid, self.u[sl], self.dfeat[sl], N, m.dtable, self.ws_enc)
                else:
                    B.dg_hashgrid_encode_bwd(m.grid, self.u[sl], self.dfeat[sl], N, m.dtable, self.ws_enc)

    def step(self, o, d, Cgt, jitter=None, foreign=None):
        self.forward(o, d, Cgt, jitter, foreign)
        self.backward()

    # -- optimiser (Sec. 5.1) -----------------------------------------------------------------
    def optimiser_step(self, iteration, total_iterations=300000, lr0=0.05, lr1=0.005, l2_weights=1e-6, check_overflow=False):
        """Adam on every resident sub-model, learning rate from the cosine schedule; consumes (clears) the gradients.
        iteration counts from 0.
        check_overflow: the back-propagated deltas are fp16 values times loss_scale; where one overflows, the weight
        gradient (and the table gradient) of that step is not finite.  With this flag the weight gradients are looked
        at first (one small device-to-host read); if any is not finite the step is dropped -- gradients cleared, no
        update, loss_scale halved -- and None is returned."""
        if check_overflow and not all(bool(torch.isfinite(self.models[p].dW).all()) for p in self.resident):
            for p in self.resident:
                self.models[p].dW.zero_()
                self.models[p].dtable.zero_()
            self.loss_scale *= 0.5
            return None
        lr = B.dg_cosine_lr(lr0, lr1, iteration, total_iterations)
        for p in self.resident:
            m = self.models[p]
            st = m.optimiser_state()
            with self._timed("dg_adam_step"):
                B.dg_adam_step(m.table.reshape(-1), m.dtable.reshape(-1), st["table_m"].reshape(-1), st["table_v"].reshape(-1), lr,
                               iteration + 1, skip_zero_grad=True)
                B.dg_adam_step(st["w_master"], m.dW, st["w_m"], st["w_v"], lr, iteration + 1, l2=l2_weights,
                               param_half=m.weights.reshape(-1))
        return lr
