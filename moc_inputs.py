"""Seeded synthetic inputs for the Mixture-of-Contexts attention layer.

This module serves BOTH the CPU oracle's tests and the HIP path's tests/bench.
It contains no arithmetic of the method itself: only token-stream layouts
(chunk offsets, shot ids, window ids, text spans) and seeded random tensors.

Layouts follow the structure of the paper's workloads (Sec. 3.2 "Content-aligned
Chunking", Sec. 4 "Baselines", App. "Wan-2.1-1.3B Experiment"): a flattened
stream of interleaved text/video pairs; per shot a caption span followed by the
shot's latent frames in time order, each frame's tokens contiguous; chunk
boundaries coincide with frame / shot / caption boundaries.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class Layout:
    """Token-stream partition handed to ``moc_chunk_meta``.

    offsets      int32 [C+1]  chunk j covers tokens [offsets[j], offsets[j+1])
    shot         int32 [C]    non-decreasing shot id per chunk
    window       int32 [C]    chunks with equal id are mutually mandatory
                              (intra-shot local window); contiguous per id
    text_spans   int32 [T,2]  token ranges [start,end) of caption spans; each a
                              union of whole chunks
    """
    name: str
    offsets: np.ndarray
    shot: np.ndarray
    window: np.ndarray
    text_spans: np.ndarray
    meta: dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return int(self.offsets[-1])

    @property
    def C(self) -> int:
        return int(self.offsets.shape[0] - 1)

    @property
    def T(self) -> int:
        return int(self.text_spans.shape[0])


def _finish(name, offs, shot, win, spans, **meta) -> Layout:
    return Layout(
        name=name,
        offsets=np.asarray(offs, dtype=np.int32),
        shot=np.asarray(shot, dtype=np.int32),
        window=np.asarray(win, dtype=np.int32),
        text_spans=np.asarray(spans, dtype=np.int32).reshape(-1, 2),
        meta=meta,
    )


def multishot_layout(n_shots: int, text_len: int, frames: int, frame_tokens: int,
                     chunk: int, window: str = "frame", name: str = "") -> Layout:
    """Regular interleaved layout: per shot [caption span | frame 0 | frame 1 ...].

    window: "chunk" (own chunk only), "frame" (all chunks of the frame) or
            "shot" (every chunk of the shot, its caption chunk included).
    Each caption span is ONE chunk. ``chunk`` must divide ``frame_tokens``.
    """
    if frame_tokens % chunk != 0:
        raise ValueError("chunk must divide frame_tokens")
    if window not in ("chunk", "frame", "shot"):
        raise ValueError(window)
    per_frame = frame_tokens // chunk
    offs, shot, win, spans = [0], [], [], []
    wid = 0
    for s in range(n_shots):
        shot_wid = wid
        if window == "shot":
            wid += 1
        if text_len > 0:
            start = offs[-1]
            offs.append(start + text_len)
            spans.append((start, start + text_len))
            shot.append(s)
            if window == "shot":
                win.append(shot_wid)
            else:
                win.append(wid)
                wid += 1
        for _f in range(frames):
            frame_wid = wid
            if window == "frame":
                wid += 1
            for _c in range(per_frame):
                offs.append(offs[-1] + chunk)
                shot.append(s)
                if window == "chunk":
                    win.append(wid)
                    wid += 1
                elif window == "frame":
                    win.append(frame_wid)
                else:
                    win.append(shot_wid)
    return _finish(name or f"{n_shots}shot_c{chunk}_{window}", offs, shot, win, spans,
                   n_shots=n_shots, text_len=text_len, frames=frames,
                   frame_tokens=frame_tokens, chunk=chunk, window=window)


def stream_layout(n_shots: int, text_len: int, video_tokens: int, chunk: int, window: str = "shot",
                  name: str = "") -> Layout:
    """Per shot [caption span | video_tokens], the video cut every ``chunk`` tokens with a ragged
    last chunk, never across a shot boundary (App. "Training Details": fixed chunk sizes over the
    flattened stream). window: "chunk" (own chunk) or "shot" (the whole shot, caption included)."""
    if window not in ("chunk", "shot"):
        raise ValueError(window)
    offs, shot, win, spans = [0], [], [], []
    wid = 0
    for s in range(n_shots):
        if text_len > 0:
            start = offs[-1]
            offs.append(start + text_len)
            spans.append((start, start + text_len))
            shot.append(s)
            win.append(wid)
            if window == "chunk":
                wid += 1
        left = video_tokens
        while left > 0:
            m = min(chunk, left)
            offs.append(offs[-1] + m)
            shot.append(s)
            win.append(wid)
            if window == "chunk":
                wid += 1
            left -= m
        if window == "shot":
            wid += 1
    return _finish(name or f"{n_shots}shot_stream_c{chunk}_{window}", offs, shot, win, spans,
                   n_shots=n_shots, text_len=text_len, video_tokens=video_tokens, chunk=chunk, window=window)


def mixed_stream_layout(n_shots: int, text_len: int, video_tokens: int, sizes: Sequence[int],
                        window: str = "shot", name: str = "") -> Layout:
    """Per shot [caption span | video_tokens] with chunks of MIXED sizes in one stream: the video of a
    shot is cut into chunks whose sizes cycle through ``sizes`` (the four sizes of the multi-shot
    training schedule side by side, App. "Training Details"; Sec. 3.2: chunk lengths are highly
    unequal), the shot's last chunk being whatever is left; shot s starts the cycle at sizes[s % len]."""
    if window not in ("chunk", "shot"):
        raise ValueError(window)
    offs, shot, win, spans = [0], [], [], []
    wid = 0
    for s in range(n_shots):
        if text_len > 0:
            start = offs[-1]
            offs.append(start + text_len)
            spans.append((start, start + text_len))
            shot.append(s)
            win.append(wid)
            if window == "chunk":
                wid += 1
        left, c = video_tokens, s
        while left > 0:
            m = min(int(sizes[c % len(sizes)]), left)
            offs.append(offs[-1] + m)
            shot.append(s)
            win.append(wid)
            if window == "chunk":
                wid += 1
            left -= m
            c += 1
        if window == "shot":
            wid += 1
    return _finish(name or f"{n_shots}shot_mixed_{window}", offs, shot, win, spans, n_shots=n_shots,
                   text_len=text_len, video_tokens=video_tokens, chunk="mixed " + "/".join(str(x) for x in sizes),
                   window=window)


def random_layout(seed: int, n_chunks: int = 12, max_len: int = 40, n_shots: int = 2,
                  text_prob: float = 0.2, window: str = "mixed") -> Layout:
    """Small irregular layout for brute-force tests: chunk lengths 1..max_len,
    several caption spans at random places, windows of random extent that stay
    inside one shot and never mix text with video unless window == "shot"."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, max_len + 1, size=n_chunks)
    offs = np.concatenate([[0], np.cumsum(lens)])
    cuts = np.sort(rng.choice(np.arange(1, n_chunks), size=min(n_shots - 1, n_chunks - 1),
                              replace=False)) if n_shots > 1 else np.array([], dtype=int)
    shot = np.searchsorted(cuts, np.arange(n_chunks), side="right")
    is_text = rng.random(n_chunks) < text_prob
    spans = []
    j = 0
    while j < n_chunks:                      # adjacent text chunks form one span
        if is_text[j]:
            e = j
            while e + 1 < n_chunks and is_text[e + 1] and rng.random() < 0.5:
                e += 1
            spans.append((int(offs[j]), int(offs[e + 1])))
            j = e + 1
        else:
            j += 1
    win = np.zeros(n_chunks, dtype=np.int64)
    wid = 0
    j = 0
    while j < n_chunks:
        if window == "chunk":
            ext = 1
        elif window == "shot":
            ext = n_chunks
        else:
            ext = int(rng.integers(1, 5))
        e = j
        while (e + 1 < n_chunks and e + 1 - j < ext and shot[e + 1] == shot[j]
               and (window == "shot" or is_text[e + 1] == is_text[j])):
            e += 1
        win[j:e + 1] = wid
        wid += 1
        j = e + 1
    return _finish(f"rand{seed}", offs, shot, win, spans, seed=seed)


# ---- the named workloads ------------------------------------------------------

def config_layout(cfg: str, window: Optional[str] = None, chunk: Optional[int] = None) -> Layout:
    if cfg == "tiny":        # 64 text + 1 shot x 4 frames x 256 tokens, chunk 64, own-chunk window
        return multishot_layout(1, 64, 4, 256, chunk or 64, window or "chunk", "tiny")
    if cfg == "single":      # 512 text + 21 frames x 1560 tokens, chunk 260, own-frame window
        return multishot_layout(1, 512, 21, 1560, chunk or 260, window or "frame", "single")
    if cfg == "eight":       # 8 x (256 text + 9 frames x 1560), chunk 260
        return multishot_layout(8, 256, 9, 1560, chunk or 260, window or "frame", "eight")
    if cfg == "sweep":       # 32 x (256 text + 9 frames x 1560), chunk in {130,260,520}
        return multishot_layout(32, 256, 9, 1560, chunk or 260, window or "frame", "sweep")
    if cfg == "short":       # single-shot training set-up: 256 text + 6,000 video tokens, chunk 256, own-chunk window
        return stream_layout(1, 256, 6000, chunk or 256, window or "chunk", "short")
    if cfg == "paper":       # multi-shot training set-up: 8 x (256 text + 14,040 video), chunk 10240 ... 1280, shot window
        return stream_layout(8, 256, 14040, chunk or 1280, window or "shot", "paper")
    if cfg == "long":        # the paper's 8-shot scale: 8 x (256 text + 22,464 video) = 181,760 tokens, chunks of mixed sizes
        return mixed_stream_layout(8, 256, 22464, (10240, 5120, 2560, 1280), window or "shot", "long")
    raise ValueError(cfg)


CONFIGS = {
    #  name      B  H   d    dtype   topk
    "tiny":   dict(B=1, H=2,  d=64,  dtype="f32",  topk=2),
    "single": dict(B=1, H=24, d=128, dtype="bf16", topk=5),
    "eight":  dict(B=1, H=24, d=128, dtype="bf16", topk=8),
    "sweep":  dict(B=1, H=24, d=128, dtype="bf16", topk=8),
    # the two training set-ups of App. "Training Details" (no causal mask in the single-shot one)
    "short":  dict(B=1, H=24, d=128, dtype="bf16", topk=3, causal=False),
    "paper":  dict(B=1, H=24, d=128, dtype="bf16", topk=5),
    # Sec. 3.3 worked example / Sec. 4: 8 shots x ~23k tokens = ~180k tokens, k=5, shot window, mixed chunk sizes
    "long":   dict(B=1, H=24, d=128, dtype="bf16", topk=5),
}


# ---- seeded tensors ----------------------------------------------------------

def randn(shape: Sequence[int], seed: int, device: str = "cpu", bf16_round: bool = True):
    """iid N(0,1) float32 tensor drawn with torch's seeded generator on `device`.
    With bf16_round the values are rounded to bf16 (nearest-even) and widened
    back, so a bf16 copy and the float32 copy hold identical values."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    x = torch.randn(*shape, generator=g, device=device, dtype=torch.float32)
    if bf16_round:
        x = x.to(torch.bfloat16).to(torch.float32)
    return x


def qkv_do(B: int, H: int, N: int, d: int, seed: int, device: str = "cpu", bf16_round: bool = True):
    """q, k, v, dO drawn in that order from consecutive seeds (S1 recipe)."""
    return tuple(randn((B, H, N, d), seed + 7919 * i, device, bf16_round) for i in range(4))


def coherent_qk(layout: Layout, B: int, H: int, d: int, seed: int, rho: float = 0.9,
                device: str = "cpu"):
    """S2 recipe: chunk-coherent q and k. Tokens of a chunk share a dominant
    component u_c (x_t = sqrt(rho) u_c + sqrt(1-rho) eps_t); the query-side
    component of chunk c is correlated with the key-side component of a seeded
    random EARLIER chunk pi(c), so retrieval has a planted target."""
    import torch
    N, C = layout.N, layout.C
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    lens = torch.from_numpy(np.diff(layout.offsets).astype(np.int64))
    chunk_of = torch.repeat_interleave(torch.arange(C), lens)
    uk = torch.randn(B, H, C, d, generator=g)
    gq = torch.randn(B, H, C, d, generator=g)
    pi = torch.tensor([int(torch.randint(0, max(c, 1), (1,), generator=g)) for c in range(C)])
    uq = 0.5 * uk[:, :, pi, :] + (0.75 ** 0.5) * gq
    eq = torch.randn(B, H, N, d, generator=g)
    ek = torch.randn(B, H, N, d, generator=g)
    q = (rho ** 0.5) * uq[:, :, chunk_of, :] + ((1 - rho) ** 0.5) * eq
    k = (rho ** 0.5) * uk[:, :, chunk_of, :] + ((1 - rho) ** 0.5) * ek
    q = q.to(torch.bfloat16).to(torch.float32).to(device)
    k = k.to(torch.bfloat16).to(torch.float32).to(device)
    return q, k
