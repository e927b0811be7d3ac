"""Device-side plumbing for a trace: the HBM frame pool, the pinned host backing store
filled with the seeded page contents, and the page-id pool of LIST launches.  Torch is
used for memory only; nothing here knows what the scheduler does with these buffers."""
import numpy as np

from .content import page_words_torch

NONE = 0xFFFFFFFF
POISON = 0x5A5A5A5A5A5A5A5A


class DeviceBuffers:
    def __init__(self, trace, fill_contents=True, device="cuda:0"):
        import torch
        self.torch, self.trace = torch, trace
        self.device = torch.device(device)
        self.wpp = trace.page_bytes // 8
        self.pool = torch.full((trace.n_frames, self.wpp), POISON, dtype=torch.int64, device=self.device)
        self.host = torch.empty((trace.n_slots, self.wpp), dtype=torch.int64, pin_memory=True)
        self.ids, self.ids_ptr = None, 0
        if trace.ids_pool.size:
            self.ids = torch.from_numpy(trace.ids_pool.view(np.int32)).to(self.device)
            self.ids_ptr = self.ids.data_ptr()
        self.pages_with_slot = (np.arange(trace.n_virtual_pages) if trace.host_slot is None
                                else np.nonzero(trace.host_slot != NONE)[0])
        if fill_contents:
            self.fill_host_store()
        else:
            self.host.fill_(1)
        torch.cuda.synchronize()

    def fill_host_store(self):
        """host[slot(p)] = initial contents of page p, generated on the device in chunks."""
        torch, trace = self.torch, self.trace
        pages = self.pages_with_slot
        identity = trace.host_slot is None
        slot = pages if identity else trace.host_slot[pages].astype(np.int64)
        step = max(1, (256 << 20) // trace.page_bytes)
        for i in range(0, pages.size, step):
            pg = torch.from_numpy(pages[i:i + step].astype(np.int64)).to(self.device)
            words = page_words_torch(pg, self.wpp)
            if identity:
                self.host[i:i + step].copy_(words)
            else:
                self.host[torch.from_numpy(np.asarray(slot[i:i + step], np.int64))] = words.cpu()

    def stamp(self, frames, idx, val):
        """pool[frames[k], idx[k]] = val[k]: what the running task writes into its pages."""
        torch = self.torch
        if len(frames) == 0:
            return
        f = torch.from_numpy(np.asarray(frames, np.int64)).to(self.device)
        i = torch.from_numpy(np.asarray(idx, np.int64)).to(self.device)
        v = torch.from_numpy(np.asarray(val, np.uint64).view(np.int64)).to(self.device)
        self.pool[f, i] = v

    def pool_words(self):
        self.torch.cuda.synchronize()
        return self.pool.cpu().numpy().view(np.uint64)

    def host_words(self):
        self.torch.cuda.synchronize()
        return self.host.numpy().view(np.uint64)

    def release(self):
        """Drop the buffers and hand cached device and pinned memory back to the system."""
        torch = self.torch
        torch.cuda.synchronize()
        self.pool = self.host = self.ids = None
        torch.cuda.empty_cache()
        empty_host = getattr(torch._C, "_host_emptyCache", None)
        if empty_host is not None:
            empty_host()
