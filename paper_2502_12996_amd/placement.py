"""Placement of caller buffers by memory class on MI355X (optional; the C ABI never allocates).

Measured on this GPU: its 288 GiB fall into three classes of 96 GiB (a third each; presumably
the ranks of the 12-high HBM3E stacks, which no interface names).  Two streams that are read
together run about 5 % faster when both lie in one class than across two (7.2-7.4 against
6.85-7.0 TB/s for two 2 GiB streams), writes behave the other way round, and the sweeps of this
library follow: the AdamW sweep with all four arrays in one class reaches 83.3-84.3 % of the HBM
peak against 79.6-82.4 % with its arrays spread over classes, the eager outer step 81.5-82.3 %
against 80.5-81 % for buffers that straddle classes.  An ordinary allocation is laid over whatever physical memory is
free, so which case a process gets is luck (one run in three is good).

`Arena` takes device memory as physical chunks through HIP's virtual memory management, maps them
side by side, tells the classes apart by timing (`diloco_sim_stream_sweep`, two read streams, every
chunk against a reference chunk), and then maps chunks of one class behind each other for each group
of buffers that stream together.  It hands out torch tensors over that memory; the memory stays the
arena's until `close()`.  Everything here is host plumbing (HIP API calls and timing of an existing
kernel); none of the method's arithmetic.  Every HIP error raises `PlacementError` before anything
is launched on the memory concerned, so a caller can fall back to ordinary allocations.
"""
from __future__ import annotations

import ctypes
from typing import Dict, List, Optional, Sequence, Tuple

CHUNK_BYTES = 2 << 30
ALIGN_BYTES = 4096            # every placed buffer starts on such a boundary
SAME_CLASS_MIN_GAIN = 0.03    # two read streams in one class run at least this much faster than across classes
                              # (measured 4.3-4.8 %; rates inside one class spread by up to 2.5 %)
CLASS_CHUNKS_MAX = 50         # no class holds more 2 GiB chunks than this (a third of 288 GiB is 48)


class PlacementError(RuntimeError):
    pass


# ------------------------------------------------------------------ pure helpers (tested on the CPU)
def split_by_rate(rates: Dict[int, float], min_gain: float = SAME_CLASS_MIN_GAIN
                  ) -> Tuple[Optional[float], List[int], List[int]]:
    """Two-stream read rates of a reference chunk against other chunks -> (threshold, same, other).

    The rates fall into a fast group (same class as the reference) and a slow one: two centres are
    fitted (2-means from the extremes) and the threshold is half-way between them, unless the
    centres lie closer than `min_gain` (relative): then there is one group only and the threshold is
    None (same = all chunks, other = [])."""
    keys = sorted(rates, key=lambda k: rates[k])
    vals = [rates[k] for k in keys]
    if len(vals) < 2 or vals[-1] <= 0.0:
        return None, list(keys), []
    # centres of the two groups by a few rounds of 2-means from the extremes
    lo, hi = vals[0], vals[-1]
    for _ in range(16):
        mid = 0.5 * (lo + hi)
        a = [v for v in vals if v <= mid]
        b = [v for v in vals if v > mid]
        if not a or not b:
            break
        nlo, nhi = sum(a) / len(a), sum(b) / len(b)
        if nlo == lo and nhi == hi:
            break
        lo, hi = nlo, nhi
    if hi - lo < min_gain * hi:
        return None, list(keys), []
    thr = 0.5 * (lo + hi)
    return thr, [k for k in keys if rates[k] > thr], [k for k in keys if rates[k] <= thr]


def plan_groups(labels: Sequence[int], groups: Sequence[int]) -> List[List[int]]:
    """Chunks for each group (sizes in chunks, in order of priority), each group from as few classes as
    possible: the class with the fewest free chunks that still holds the whole group, else the largest
    class first and the rest from the next.  Chunks labelled -1 (mixed) are used last.  Raises
    PlacementError if the chunks do not suffice."""
    free: Dict[int, List[int]] = {}
    for i, lab in enumerate(labels):
        free.setdefault(lab, []).append(i)
    out = []
    for need in groups:
        if need > sum(len(v) for v in free.values()):
            raise PlacementError(f"a group of {need} chunks does not fit what is left")
        proper = {c: v for c, v in free.items() if c >= 0}
        fits = [c for c, v in proper.items() if len(v) >= need]
        order = ([min(fits, key=lambda c: len(proper[c]))] if fits
                 else sorted(proper, key=lambda c: -len(proper[c]))) + [c for c in free if c < 0]
        got: List[int] = []
        for c in order + [c for c in proper if c not in order]:
            take = free[c][:need - len(got)]
            free[c] = free[c][len(take):]
            got += take
            if len(got) == need:
                break
        out.append(got)
    return out


def label_chunks(n: int, measure, max_classes: int = 8, min_members: int = 5,
                 class_max: int = CLASS_CHUNKS_MAX) -> Tuple[List[int], List[Dict[int, float]]]:
    """Labels 0, 1, ... (-1: no class) for n chunks.  measure(ref, rest) returns the two-stream read rate
    of chunk `ref` with every chunk of `rest`.  One reference per class: the first chunk without a
    label; the chunks that run fast with it share its class.  A reference with which more chunks run
    fast than a class can hold straddles two classes and gets -1, as do, in the end, the chunks of
    classes with fewer than `min_members` members (straddling chunks, disturbed measurements).
    Returns (labels, the rates of every round)."""
    labels: List[Optional[int]] = [None] * n
    history: List[Dict[int, float]] = []
    classes = 0
    while None in labels and classes < max_classes:
        ref = labels.index(None)
        rest = [k for k in range(n) if labels[k] is None and k != ref]
        rates = measure(ref, rest) if rest else {}
        history.append(rates)
        _, same, _ = split_by_rate(rates)
        if len(same) + 1 > class_max:
            labels[ref] = -1
            continue
        labels[ref] = classes
        for k in same:
            labels[k] = classes
        classes += 1
    sizes: Dict[int, int] = {}
    for lab in labels:
        if lab is not None and lab >= 0:
            sizes[lab] = sizes.get(lab, 0) + 1
    keep = {c: i for i, c in enumerate(sorted(c for c, m in sizes.items() if m >= min(min_members, n)))}
    return [keep.get(lab, -1) if lab is not None else -1 for lab in labels], history


# ------------------------------------------------------------------ HIP virtual memory management
class _Loc(ctypes.Structure):
    _fields_ = [("type", ctypes.c_int), ("id", ctypes.c_int)]


class _AllocFlags(ctypes.Structure):
    _fields_ = [("compressionType", ctypes.c_ubyte), ("gpuDirectRDMACapable", ctypes.c_ubyte),
                ("usage", ctypes.c_ushort)]


class _Prop(ctypes.Structure):       # hipMemAllocationProp
    _fields_ = [("type", ctypes.c_int), ("requestedHandleType", ctypes.c_int), ("location", _Loc),
                ("win32HandleMetaData", ctypes.c_void_p), ("allocFlags", _AllocFlags)]


class _Access(ctypes.Structure):     # hipMemAccessDesc
    _fields_ = [("location", _Loc), ("flags", ctypes.c_int)]


_PINNED, _DEVICE, _READ_WRITE = 1, 1, 3   # hipMemAllocationTypePinned, hipMemLocationTypeDevice, ...ProtReadWrite


def _runtime():
    """The HIP runtime this process already uses (the one torch loaded), with the signatures needed."""
    path = None
    with open("/proc/self/maps") as maps:
        for line in maps:
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
    if path is None:
        raise PlacementError("no HIP runtime is loaded in this process")
    hip = ctypes.CDLL(path)
    vp, sz, ull = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_ulonglong
    hip.hipMemCreate.argtypes = [ctypes.POINTER(vp), sz, ctypes.POINTER(_Prop), ull]
    hip.hipMemAddressReserve.argtypes = [ctypes.POINTER(vp), sz, sz, vp, ull]
    hip.hipMemMap.argtypes = [vp, sz, sz, vp, ull]
    hip.hipMemSetAccess.argtypes = [vp, sz, ctypes.POINTER(_Access), sz]
    hip.hipMemUnmap.argtypes = [vp, sz]
    hip.hipMemRelease.argtypes = [vp]
    hip.hipMemAddressFree.argtypes = [vp, sz]
    return hip


class _Span:
    """__cuda_array_interface__ over a mapped address range (bytes)."""

    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


class Arena:
    """Physical chunks of device memory, classified, and mapped class by class for groups of buffers.

    arena = Arena(device=0)                   # takes chunks: all free memory but `keep_free`, or `max_chunks`
    arena.classify()                          # labels every chunk (0, 1, 2; -1 = straddles two classes)
    bufs = arena.place([[("theta", nbytes), ("m1", nbytes)], [("state", nbytes)]])   # uint8 tensors
    arena.release_rest()                      # chunks not placed go back to the driver
    ... use bufs["theta"].view(torch.float32) ...
    arena.close()                             # after the last use of the tensors: unmaps and frees
    (also a context manager: `with Arena() as arena: ...` closes on the way out)
    """

    def __init__(self, device: int = 0, chunk_bytes: int = CHUNK_BYTES, keep_free: int = 8 << 30,
                 max_chunks: Optional[int] = None):
        import torch
        self.torch = torch
        self.device = device
        self.chunk = int(chunk_bytes)
        if self.chunk <= 0 or self.chunk % (2 << 20):
            raise ValueError("chunk_bytes must be a positive multiple of 2 MiB")
        torch.cuda.init()
        torch.zeros(1, device=f"cuda:{device}")
        self.hip = _runtime()
        self.handles: List[Optional[ctypes.c_void_p]] = []
        self.labels: List[int] = []
        self.scan_va: Optional[int] = None
        self.ranges: List[Tuple[int, int]] = []       # (address, bytes) of the placed groups
        self.placed: set = set()
        self.rates: List[Dict[int, float]] = []
        prop = _Prop(_PINNED, 0, _Loc(_DEVICE, device), None, _AllocFlags(0, 0, 0))
        with torch.cuda.device(device):
            free, _ = torch.cuda.mem_get_info()
            count = max(0, (free - keep_free) // self.chunk)
            if max_chunks is not None:
                count = min(count, max_chunks)
            for _ in range(int(count)):
                h = ctypes.c_void_p()
                if self.hip.hipMemCreate(ctypes.byref(h), self.chunk, ctypes.byref(prop), 0) != 0:
                    break                              # the driver has no more: go on with what there is
                self.handles.append(h)
            if not self.handles:
                raise PlacementError("no device memory could be taken in chunks")
            try:
                self.scan_va = self._map(list(range(len(self.handles))))
            except PlacementError:
                self.close()
                raise

    # -- mapping
    def _check(self, rc: int, what: str) -> None:
        if rc != 0:
            raise PlacementError(f"{what}: HIP error {rc}")

    def _map(self, chunks: Sequence[int]) -> int:
        """Reserve an address range and map the chunks into it, in order; returns its address."""
        size = len(chunks) * self.chunk
        va = ctypes.c_void_p()
        # aligned like a chunk, so that the page tables can describe a chunk by large fragments
        self._check(self.hip.hipMemAddressReserve(ctypes.byref(va), size, self.chunk, None, 0),
                    "hipMemAddressReserve")
        done = 0
        try:
            for slot, c in enumerate(chunks):
                self._check(self.hip.hipMemMap(va.value + slot * self.chunk, self.chunk, 0, self.handles[c], 0),
                            "hipMemMap")
                done += 1
            acc = _Access(_Loc(_DEVICE, self.device), _READ_WRITE)
            self._check(self.hip.hipMemSetAccess(va.value, size, ctypes.byref(acc), 1), "hipMemSetAccess")
        except PlacementError:
            if done:
                self.hip.hipMemUnmap(va.value, done * self.chunk)
            self.hip.hipMemAddressFree(va.value, size)
            raise
        return va.value

    def _unmap(self, va: int, size: int) -> None:
        self.torch.cuda.synchronize(self.device)
        self._check(self.hip.hipMemUnmap(va, size), "hipMemUnmap")
        self._check(self.hip.hipMemAddressFree(va, size), "hipMemAddressFree")

    def _tensor(self, ptr: int, nbytes: int):
        return self.torch.as_tensor(_Span(ptr, nbytes), device=f"cuda:{self.device}")

    # -- classes
    def _pair_rate(self, binding, i: int, j: int, reps: int) -> float:
        """GB/s of chunks i and j read together as two streams (best of `reps`)."""
        torch = self.torch
        lo, hi = min(i, j), max(i, j)
        q = self.chunk // 4
        span = self._tensor(self.scan_va + lo * self.chunk, (hi - lo + 1) * self.chunk).view(torch.float32)
        rows = span.as_strided((2, q), ((hi - lo) * q, 1))
        binding.sim_stream_sweep(rows, binding.SWEEP_READ)
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            binding.sim_stream_sweep(rows, binding.SWEEP_READ)
            e1.record()
            torch.cuda.synchronize(self.device)
            ms = e0.elapsed_time(e1)
            best = ms if best is None or ms < best else best
        return 2.0 * self.chunk / best / 1e6

    def classify(self, reps: int = 5, max_classes: int = 8, min_members: int = 5) -> List[int]:
        """Label every chunk with its class by timing it against one reference chunk per class.  A class
        of fewer than `min_members` chunks is noise (a chunk that straddles two classes, a disturbed
        measurement): its chunks are labelled -1 like the straddling references."""
        from . import binding
        torch = self.torch
        if self.scan_va is None:
            raise PlacementError("the chunks are no longer mapped side by side")
        n = len(self.handles)
        with torch.cuda.device(self.device):
            whole = self._tensor(self.scan_va, n * self.chunk)
            for k in range(n):                       # physical memory comes as it is: give the reads finite values
                whole[k * self.chunk:(k + 1) * self.chunk].zero_()
            del whole
            torch.cuda.synchronize(self.device)
            def measure(ref, rest):
                return {k: self._pair_rate(binding, ref, k, reps) for k in rest}
            self.labels, self.rates = label_chunks(
                n, measure, max_classes, min_members,
                CLASS_CHUNKS_MAX * max(1, CHUNK_BYTES // self.chunk))
        return self.labels

    # -- buffers
    def place(self, groups: Sequence[Sequence[Tuple[str, int]]]) -> Dict[str, "object"]:
        """Map one address range per group, from chunks of one class where they suffice, and carve the
        group's buffers out of it one behind the other.  groups: [[(name, bytes), ...], ...], the most
        important group first.  Returns name -> uint8 tensor of that many bytes."""
        if not self.labels:
            self.labels = [0] * len(self.handles)
        if self.scan_va is not None:
            self._unmap(self.scan_va, len(self.handles) * self.chunk)
            self.scan_va = None
        sizes = []
        for g in groups:
            total = sum(-(-int(b) // ALIGN_BYTES) * ALIGN_BYTES for _, b in g)
            sizes.append(-(-total // self.chunk))
        avail = [lab if (i not in self.placed and self.handles[i] is not None) else None
                 for i, lab in enumerate(self.labels)]
        idx = [i for i, lab in enumerate(avail) if lab is not None]
        plan = plan_groups([avail[i] for i in idx], sizes)
        out: Dict[str, object] = {}
        for g, chunks in zip(groups, plan):
            chunks = [idx[c] for c in chunks]
            va = self._map(chunks)
            self.ranges.append((va, len(chunks) * self.chunk))
            self.placed.update(chunks)
            off = 0
            for name, nbytes in g:
                out[name] = self._tensor(va + off, int(nbytes))
                off += -(-int(nbytes) // ALIGN_BYTES) * ALIGN_BYTES
        return out

    def release_rest(self) -> None:
        """Chunks that no placed buffer uses go back to the driver."""
        if self.scan_va is not None:
            self._unmap(self.scan_va, len(self.handles) * self.chunk)
            self.scan_va = None
        for i, h in enumerate(self.handles):
            if h is not None and i not in self.placed:
                self._check(self.hip.hipMemRelease(h), "hipMemRelease")
                self.handles[i] = None

    def close(self) -> None:
        """Unmap and free everything.  No tensor handed out may be used afterwards."""
        if getattr(self, "hip", None) is None:
            return
        self.torch.cuda.synchronize(self.device)
        if self.scan_va is not None:
            self.hip.hipMemUnmap(self.scan_va, len(self.handles) * self.chunk)
            self.hip.hipMemAddressFree(self.scan_va, len(self.handles) * self.chunk)
            self.scan_va = None
        for va, size in self.ranges:
            self.hip.hipMemUnmap(va, size)
            self.hip.hipMemAddressFree(va, size)
        self.ranges = []
        for i, h in enumerate(self.handles):
            if h is not None:
                self.hip.hipMemRelease(h)
                self.handles[i] = None
        self.placed = set()

    def __enter__(self) -> "Arena":
        return self

    def __exit__(self, *exc) -> None:
        self.close()

    def summary(self) -> Dict[str, object]:
        counts: Dict[int, int] = {}
        for lab in self.labels:
            counts[lab] = counts.get(lab, 0) + 1
        return {"chunk_bytes": self.chunk, "chunks": len(self.labels),
                "chunks_per_class": {str(k): v for k, v in sorted(counts.items())},
                "placed_chunks": len(self.placed)}


def main() -> None:
    """python -m paper_2502_12996_amd.placement: take the free device memory, label its chunks, print the map."""
    arena = Arena()
    try:
        labels = arena.classify()
        print(f"{len(labels)} chunks of {arena.chunk >> 20} MiB; chunks per class: {arena.summary()['chunks_per_class']}")
        print("classes in mapping order ('.' = set aside):",
              "".join("abcdefgh"[lab] if 0 <= lab < 8 else "." for lab in labels))
        for k, rates in enumerate(arena.rates):
            thr, same, other = split_by_rate(rates)
            vals = sorted(rates.values())
            if not vals:
                continue
            if thr is None:
                print(f"reference {k}: {len(vals)} chunks, one group, {vals[0]:.0f} .. {vals[len(vals) // 2]:.0f} .. "
                      f"{vals[-1]:.0f} GB/s")
            else:
                fast = sorted(rates[c] for c in same)
                slow = sorted(rates[c] for c in other)
                print(f"reference {k}: {len(fast)} chunks read with it at {fast[0]:.0f} .. {fast[len(fast) // 2]:.0f} .. "
                      f"{fast[-1]:.0f} GB/s, {len(slow)} at {slow[0]:.0f} .. {slow[len(slow) // 2]:.0f} .. {slow[-1]:.0f} GB/s")
    finally:
        arena.close()


if __name__ == "__main__":
    main()
