"""Harness plumbing shared by the benchmark and the tests: turns a synthetic Step into pool
images, uploads them with torch (device memory and pinned host memory only) and drives the
library through its binding.  No arithmetic of the method lives here."""
import numpy as np

from . import workload as wl


def poison_value(dtype):
    return np.float32(np.nan) if dtype == "f32" else (0x7E00 if dtype == "f16" else 0x7FC0)


def build_pools(step, poison_rest=False, into=None):
    """Device-tier and host-tier pool images ([n_blocks, block_elems] storage arrays) at
    the start of the step: blocks on the swap-in list have their content on the host tier
    and poison on the device tier.  `into=(dev, host)` adds the step to existing images
    (several steps with disjoint blocks in one pool)."""
    cfg = step.cfg
    sd = wl.storage_dtype(cfg.dtype)
    if into is None:
        dev = np.zeros((cfg.n_dev_blocks, cfg.block_elems), dtype=sd)
        host = np.zeros((cfg.n_host_blocks, cfg.block_elems), dtype=sd)
        if poison_rest:
            dev[:] = poison_value(cfg.dtype)
    else:
        dev, host = into
    dev[step.content_ids] = step.content
    if len(step.swap_in_dev):
        host[step.swap_in_host] = dev[step.swap_in_dev]
        dev[step.swap_in_dev] = poison_value(cfg.dtype)
    return dev, host


def resident_pool(step):
    """Device pool image with every needed block resident (swap already done)."""
    cfg = step.cfg
    dev = np.zeros((cfg.n_dev_blocks, cfg.block_elems), dtype=wl.storage_dtype(cfg.dtype))
    dev[step.content_ids] = step.content
    return dev




# ------------------------------------------------------------------ GPU plumbing (torch = memory only)
def to_dev(a, pin=False):
    import torch
    a = np.ascontiguousarray(a)
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a)
    if pin:
        return t.pin_memory()
    return t.cuda()


def to_np(t, like_dtype):
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if like_dtype == np.uint16 else a


class GpuPool:
    """The two tiers as torch tensors (device memory / pinned host memory) plus the flpool handle."""

    def __init__(self, cfg, dev_img, host_img):
        from . import flpool
        self.cfg = cfg
        self.sd = wl.storage_dtype(cfg.dtype)
        self.dev = to_dev(dev_img)
        self.host = to_dev(host_img, pin=True)
        self.pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, dev_img.shape[0], host_img.shape[0],
                                block_tokens=cfg.block_tokens, dev=self.dev, host=self.host)


class GpuStep:
    """Uploads a synthetic Step; owns (or shares) the pool it runs on."""

    def __init__(self, step, dev_img=None, host_img=None, gpool=None):
        import torch
        cfg = step.cfg
        self.step, self.cfg = step, cfg
        self.gpool = gpool if gpool is not None else GpuPool(cfg, dev_img, host_img)
        self.sd, self.dev, self.host, self.pool = self.gpool.sd, self.gpool.dev, self.gpool.host, self.gpool.pool
        self.kv_tables = to_dev(step.kv_tables)
        self.lora_tables = to_dev(step.lora_tables)
        self.token_adapter = to_dev(step.token_adapter)
        self.rank = to_dev(step.rank)
        self.scale = to_dev(step.scale)
        self.proj = {name: {k: to_dev(getattr(pr, k)) for k in ("a_tab_off", "a_row_base", "b_tab_off", "b_row_base")}
                     for name, pr in step.proj.items()}
        self.acts = {k: to_dev(v) for k, v in step.acts.items()}
        self.torch = torch

    def dev_image(self):
        self.torch.cuda.synchronize()
        return to_np(self.dev, self.sd)

    def host_image(self):
        self.torch.cuda.synchronize()
        return to_np(self.host, self.sd)

    def lora(self, names, x_key="x", w_base=None, static=False):
        """Run flp_lora_apply_paged for the named projections on copies of the base terms; returns storage arrays.
        `w_base`: optional dict name -> device tensor [d_in, d_out]; y then starts as garbage and is overwritten.
        `static`: call flp_lora_apply_paged_static instead (intermediates in the library's fixed scratch array)."""
        st = self.step
        ys = {n: self.acts["base_" + n].clone() for n in names}
        projs = [dict(y=ys[n], d_out=st.proj[n].d_out, **self.proj[n]) for n in names]
        if w_base:
            for pj, n in zip(projs, names):
                pj["w_base"] = w_base[n]
        x = self.acts[x_key]
        self.pool.lora_apply_paged(x, self.token_adapter, self.rank, self.scale, self.lora_tables, projs,
                                   n_tokens=st.n_tokens, d_in=x.shape[1], n_adapters=len(st.rank),
                                   max_rank=int(max(1, st.rank.max())), static=static)
        self.torch.cuda.synchronize()
        return {n: to_np(ys[n], self.sd) for n in names}

    def attention(self, append=True, q_key="q"):
        st, cfg = self.step, self.cfg
        q = self.acts[q_key]
        out = self.torch.zeros_like(q)
        self.pool.paged_prefix_attention(q, out, st.cu_new, st.prefix_len, self.kv_tables, cfg.n_q_heads,
                                         k_new=self.acts["k_new"] if append else None,
                                         v_new=self.acts["v_new"] if append else None)
        self.torch.cuda.synchronize()
        return to_np(out, self.sd)


# ------------------------------------------------------------------ large pools: sparse images
def compact_step(step):
    """Pool image that holds only the step's touched blocks, with the tables renumbered to
    match (block id -> row of `step.content`).  Lets the oracle follow a step whose pool is
    too large to mirror on the host; relabelling blocks changes no result."""
    n = int(step.content_ids.max()) + 1 if len(step.content_ids) else 0
    remap = np.full(n, -1, dtype=np.int64)
    remap[step.content_ids] = np.arange(len(step.content_ids))
    kv = np.where(step.kv_tables >= 0, remap[np.maximum(step.kv_tables, 0)], -1).astype(np.int32)
    lt = remap[step.lora_tables].astype(np.int32)
    return step.content.copy(), kv, lt


class SparseGpuPool:
    """Tiers of the full size on the GPU machine (device tier left uninitialised except for the
    step's blocks), for pools far larger than host memory."""

    def __init__(self, step, n_dev_blocks=None, n_host_blocks=None):
        import torch
        from . import flpool
        cfg = step.cfg
        self.cfg, self.sd = cfg, wl.storage_dtype(cfg.dtype)
        nd = cfg.n_dev_blocks if n_dev_blocks is None else n_dev_blocks
        nh = cfg.n_host_blocks if n_host_blocks is None else n_host_blocks
        tdt = torch.float32 if cfg.dtype == "f32" else torch.int16
        self.dev = torch.empty((nd, cfg.block_elems), dtype=tdt, device="cuda")
        self.host = torch.zeros((nh, cfg.block_elems), dtype=tdt).pin_memory()
        self.pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, nd, nh, block_tokens=cfg.block_tokens,
                                dev=self.dev, host=self.host)
        swapped = np.isin(step.content_ids, step.swap_in_dev)
        keep = np.flatnonzero(~swapped)
        for lo in range(0, len(keep), 1024):
            sel = keep[lo:lo + 1024]
            self.dev[torch.from_numpy(step.content_ids[sel].astype(np.int64)).cuda()] = to_dev(step.content[sel])
        row_of = {int(b): r for r, b in enumerate(step.content_ids)}
        host_np = self.host.numpy()
        for h, d in zip(step.swap_in_host, step.swap_in_dev):
            host_np[h] = step.content[row_of[int(d)]].view(host_np.dtype)
        if len(step.swap_in_dev):       # the device copies of swapped blocks start as poison
            idx = torch.from_numpy(step.swap_in_dev.astype(np.int64)).cuda()
            self.dev[idx] = int(np.array(poison_value(cfg.dtype)).astype(np.int64)) if cfg.dtype != "f32" else float("nan")

    def rows(self, ids):
        """Device blocks `ids` as a storage array."""
        import torch
        torch.cuda.synchronize()
        out = self.dev[torch.from_numpy(np.asarray(ids).astype(np.int64)).cuda()]
        return to_np(out, self.sd)
