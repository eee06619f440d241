"""Plumbing around the C ABI for tests, the smoke check and the benchmark: PyTorch lends the
device memory and the stream, this module marshals a workload description into hop_* calls and
reads ring slots back.  No arithmetic of the method happens here."""
import torch

from . import hop, inputs


class Session:
    """One hop_ctx plus the torch tensors that back it."""

    def __init__(self, c, device="cuda:0"):
        self.c = c
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        # synthetic gradients: up to sixteen waves' worth generated back to back (the mix runs slower right behind
        # the arithmetic-bound generator), one buffer per worker and wave, as far as a quarter of the free memory
        # (at most 64 GiB) holds them
        ahead = c.get("grad_ahead", 16 if c["model"] == "synth" else 1)
        if "grad_ahead" not in c and ahead > 1:
            room = min(torch.cuda.mem_get_info(self.dev)[0] // 4, 64 << 30)
            while ahead > 1 and c["N"] * ahead * (c["d"] + 128) * 4 > room:
                ahead //= 2
        self.opts = hop.make_opts(max_ig=c["max_ig"], skip_on=c["skip_on"], max_skip=c["max_skip"],
                                  trigger=c["trigger"], lr=c["lr"], lam=c["lam"], batch=c["batch"],
                                  seed=c["seed"], loss=c.get("loss", 0), momentum=c.get("momentum", 0.0),
                                  max_latency=c.get("max_latency", 0), serial=c.get("serial", False),
                                  notify_ack=c.get("notify_ack", False), grad_ahead=ahead)
        self.N, self.d = c["N"], c["d"]
        need = hop.hop_arena_bytes(self.N, self.d, c["s"], c["b"], self.opts)
        self.arena = torch.zeros(need // 4, dtype=torch.float32, device=self.dev)
        assert self.arena.data_ptr() % 256 == 0
        self.stream = torch.cuda.current_stream().cuda_stream
        row_ptr, col = inputs.to_csr(c["in_nbrs"])
        self.ctx = hop.hop_init(row_ptr, col, c["W"], self.N, self.d, c["s"], c["b"], self.opts,
                                self.arena.data_ptr(), need, self.stream)
        self.D, self.stride = hop.hop_layout(self.d, c["s"], self.opts)
        self.keep = []
        self.sched = None
        self.workspace = None

    def view(self, ptr, n):
        off = (ptr - self.arena.data_ptr()) // 4
        return self.arena[off:off + n]

    def slot(self, worker, slot):
        return self.view(hop.hop_slot(self.ctx, worker, slot), self.d)

    def ring_snapshot(self):
        """[N, D, d] numpy copy of every ring slot."""
        r = self.arena[: self.N * self.D * self.stride].view(self.N, self.D, self.stride)[:, :, : self.d]
        return r.cpu().numpy()

    def upload_rings(self, rings):
        """Overwrite every ring slot with a [N, D, d] fp32 numpy array."""
        r = self.arena[: self.N * self.D * self.stride].view(self.N, self.D, self.stride)[:, :, : self.d]
        r.copy_(torch.from_numpy(rings).to(self.dev))

    def upload_vel(self, vel):
        v = self.arena[self.arena.numel() - self.N * self.stride:].view(self.N, self.stride)[:, : self.d]
        v.copy_(torch.from_numpy(vel).to(self.dev))

    def vel_snapshot(self):
        """[N, d] numpy copy of the velocities (contexts with momentum: the arena's last N slots)."""
        v = self.arena[self.arena.numel() - self.N * self.stride:].view(self.N, self.stride)[:, : self.d]
        return v.cpu().numpy()

    def params(self):
        out, its = [], []
        for i in range(self.N):
            p, it = hop.hop_params(self.ctx, i)
            out.append(self.view(p, self.d))
            its.append(it)
        return out, its

    def set_params(self, p0):
        p0 = p0.to(self.dev).contiguous()
        self.keep.append(p0)
        hop.hop_set_params(self.ctx, p0.data_ptr(), int(p0.dim() == 2), 1)

    def set_dense(self, X, y):
        for i in range(self.N):
            Xi, yi = X[i].to(self.dev).contiguous(), y[i].to(self.dev).contiguous()
            self.keep += [Xi, yi]
            hop.hop_set_data_dense(self.ctx, i, Xi.data_ptr(), yi.data_ptr(), Xi.shape[0])
        hop.hop_set_grad_source(self.ctx, hop.HOP_GRAD_SVM_DENSE)

    def set_csr(self, data):
        for i in range(self.N):
            rp, col, val, y = [t.to(self.dev).contiguous() for t in data[i]]
            self.keep += [rp, col, val, y]
            hop.hop_set_data_csr(self.ctx, i, rp.data_ptr(), col.data_ptr(), val.data_ptr(), y.data_ptr(),
                                 rp.shape[0] - 1)
        hop.hop_set_grad_source(self.ctx, hop.HOP_GRAD_SVM_CSR)

    def simulate(self, K=None):
        c = self.c
        self.sched = hop.hop_simulate(self.ctx, c["K"] if K is None else K, c["delay_kind"], c["mult"])
        need = hop.hop_schedule_bytes(self.sched)              # descriptors live in memory torch lends
        self.workspace = torch.empty(need, dtype=torch.uint8, device=self.dev)
        assert self.workspace.data_ptr() % 256 == 0
        hop.hop_schedule_bind(self.ctx, self.sched, self.workspace.data_ptr(), need)
        return self.sched

    def step(self, wb=0, we=-1):
        hop.hop_step(self.ctx, self.sched, wb, we)

    def sync(self):
        torch.cuda.synchronize(self.dev)

    def coef(self, record):
        """Hinge coefficients of a STEP record as a numpy array (after its wave has run)."""
        self.sync()
        return hop.hop_download(hop.hop_coef(self.ctx, self.sched, record), self.c["batch"], self.stream)

    def close(self):
        self.sync()
        if self.sched is not None:
            self.sched.free()
            self.sched = None
        hop.hop_destroy(self.ctx)
        self.keep = []
        self.arena = None
        self.workspace = None


def make_data(c, device="cpu"):
    """Synthetic inputs of a config: (p0, data) with data a per-worker list."""
    seed = c["seed"]
    p0 = inputs.initial_params(seed, c["d"], 0.01, device)
    if c["model"] == "dense":
        ws = inputs.hidden_w(seed, c["d"], device)
        Xy = [inputs.dense_svm_data(seed, i, c["rows"], c["d"], ws, device) for i in range(c["N"])]
        return p0, ([x for x, _ in Xy], [y for _, y in Xy])
    if c["model"] == "csr":
        ws = inputs.hidden_w(seed, c["d"], device)
        return p0, [inputs.csr_svm_data(seed, i, c["rows"], c["d"], c["nnz"], c["zipf_a"], ws, device)
                    for i in range(c["N"])]
    return p0, None
