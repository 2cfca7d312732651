"""Seeded synthetic camera frames and token embeddings.

The paper evaluates on simulator and robot camera streams (Sec. 4.2) that are
not available here; these generators reproduce their shape (H x W x 3 uint8
frames cut into p x p patches, Sec. 3.2) and their structure (mostly static
background, a small changing region).
"""
import numpy as np


def frame_pair(H, W, patch, n_redraw, seed, jitter=2):
    """Two adjacent frames: frame t-1 is uniform random uint8; frame t copies it,
    re-draws `n_redraw` randomly chosen patches and adds integer noise in
    [-jitter, jitter] (clipped to [0, 255]) to all the others.

    Returns (prev, cur, redrawn) with redrawn a bool vector over the N*N patches
    in raster order.
    """
    rng = np.random.default_rng(seed)
    gh, gw = H // patch, W // patch
    prev = rng.integers(0, 256, size=(H, W, 3), dtype=np.uint8)
    noise = rng.integers(-jitter, jitter + 1, size=(H, W, 3)) if jitter > 0 else 0
    cur = np.clip(prev.astype(np.int64) + noise, 0, 255).astype(np.uint8)
    redrawn = np.zeros(gh * gw, dtype=bool)
    redrawn[rng.choice(gh * gw, size=n_redraw, replace=False)] = True
    fresh = rng.integers(0, 256, size=(H, W, 3), dtype=np.uint8)
    for idx in np.flatnonzero(redrawn):
        r, c = divmod(int(idx), gw)
        sl = (slice(r * patch, (r + 1) * patch), slice(c * patch, (c + 1) * patch))
        cur[sl] = fresh[sl]
    return prev, cur, redrawn


def moving_box_stream(H, W, n_frames, seed, box=48, step=6, noise=0):
    """A stream of frames: a fixed random-textured background and a
    random-textured box of `box` x `box` pixels that moves `step` pixels per
    frame along a seeded bouncing path.  Optional +-noise sensor noise.

    Returns uint8 [n_frames, H, W, 3].
    """
    rng = np.random.default_rng(seed)
    bg = rng.integers(32, 224, size=(H, W, 3), dtype=np.uint8)
    tex = rng.integers(0, 256, size=(box, box, 3), dtype=np.uint8)
    x, y = int(rng.integers(0, W - box)), int(rng.integers(0, H - box))
    dx, dy = (step if rng.random() < 0.5 else -step), 0
    frames = np.empty((n_frames, H, W, 3), dtype=np.uint8)
    for t in range(n_frames):
        f = bg.copy()
        f[y:y + box, x:x + box] = tex
        if noise > 0:
            f = np.clip(f.astype(np.int64) + rng.integers(-noise, noise + 1, size=f.shape),
                        0, 255).astype(np.uint8)
        frames[t] = f
        if rng.random() < 0.15:  # turn now and then
            dx, dy = ((0, step if rng.random() < 0.5 else -step) if dy == 0
                      else (step if rng.random() < 0.5 else -step, 0))
        nx, ny = x + dx, y + dy
        if nx < 0 or nx > W - box:
            dx = -dx
            nx = x + dx
        if ny < 0 or ny > H - box:
            dy = -dy
            ny = y + dy
        x, y = nx, ny
    return frames


def noisy_scene_stream(H, W, n_frames, seed, patch=14, noise=8, n_distractors=3, lo=16, hi=80,
                       box=48, step=6):
    """A stream in the manner of the paper's real-robot setting (Sec. 4.4): a dim static
    textured background (pixel values in [lo, hi)), sensor noise of +-`noise` on every
    pixel of every frame, one box of `box` px moving `step` px per frame (the
    manipulator) and `n_distractors` smaller boxes wandering independently (moving
    distractors in the background).  With lo > noise no background pixel is clipped.

    Returns (frames uint8 [n_frames, H, W, 3], touched bool [n_frames, n_patches]) where
    touched[t, i] says that a box overlaps patch i (raster order) in frame t.
    """
    rng = np.random.default_rng(seed)
    gh, gw = H // patch, W // patch
    bg = rng.integers(lo, hi, size=(H, W, 3), dtype=np.uint8)
    sizes = [box] + [max(patch, box // 2)] * n_distractors
    tex = [rng.integers(0, 256, size=(b, b, 3), dtype=np.uint8) for b in sizes]
    pos = [[int(rng.integers(0, W - b)), int(rng.integers(0, H - b))] for b in sizes]
    vel = []
    for k, b in enumerate(sizes):
        s = step if k == 0 else int(rng.integers(1, step + 1))
        vel.append([s if rng.random() < 0.5 else -s, 0] if rng.random() < 0.5
                   else [0, s if rng.random() < 0.5 else -s])
    frames = np.empty((n_frames, H, W, 3), dtype=np.uint8)
    touched = np.zeros((n_frames, gh * gw), dtype=bool)
    for t in range(n_frames):
        f = bg.copy()
        for k, b in enumerate(sizes):
            x, y = pos[k]
            f[y:y + b, x:x + b] = tex[k]
            r0, r1 = y // patch, min(gh - 1, (y + b - 1) // patch)
            c0, c1 = x // patch, min(gw - 1, (x + b - 1) // patch)
            m = touched[t].reshape(gh, gw)
            m[r0:r1 + 1, c0:c1 + 1] = True
        if noise > 0:
            f = np.clip(f.astype(np.int64) + rng.integers(-noise, noise + 1, size=f.shape),
                        0, 255).astype(np.uint8)
        frames[t] = f
        for k, b in enumerate(sizes):
            if rng.random() < 0.2:  # change direction now and then
                s = max(abs(vel[k][0]), abs(vel[k][1]))
                vel[k] = ([s if rng.random() < 0.5 else -s, 0] if rng.random() < 0.5
                          else [0, s if rng.random() < 0.5 else -s])
            for ax, lim in ((0, W - b), (1, H - b)):
                n = pos[k][ax] + vel[k][ax]
                if n < 0 or n > lim:
                    vel[k][ax] = -vel[k][ax]
                    n = pos[k][ax] + vel[k][ax]
                pos[k][ax] = n
    return frames, touched


def two_view_stream(H, W, n_frames, seed, pan=5):
    """Two camera views per step, stacked into one frame of 2H x W pixels (so that the
    patches in raster order are view 0's followed by view 1's): on top a fixed
    third-person view (`moving_box_stream`: mostly static), below it a wrist-camera view
    that moves with the arm: a window panning `pan` pixels per frame over a larger
    random texture, where next to nothing stays in place (Sec. 4.3 on dynamic viewpoints).

    Returns uint8 [n_frames, 2H, W, 3].
    """
    rng = np.random.default_rng(seed + 1000)
    top = moving_box_stream(H, W, n_frames, seed)
    canvas = rng.integers(0, 256, size=(H + 2 * pan * n_frames + 2, W + 2 * pan * n_frames + 2, 3),
                          dtype=np.uint8)
    x = y = pan * n_frames
    frames = np.empty((n_frames, 2 * H, W, 3), dtype=np.uint8)
    for t in range(n_frames):
        frames[t, :H] = top[t]
        frames[t, H:] = canvas[y:y + H, x:x + W]
        dx, dy = [(pan, 0), (-pan, 0), (0, pan), (0, -pan)][int(rng.integers(0, 4))]
        x, y = x + dx, y + dy
    return frames


def patch_pixels(frame, patch):
    """[H, W, 3] uint8 -> [N*N, 3*p*p] uint8, patches in raster order."""
    H, W, C = frame.shape
    gh, gw = H // patch, W // patch
    x = frame.reshape(gh, patch, gw, patch, C).transpose(0, 2, 1, 3, 4)
    return np.ascontiguousarray(x).reshape(gh * gw, patch * patch * C)


def projection_matrix(d_model, patch, seed):
    """Stand-in for the vision encoder: a fixed random linear map 3p^2 -> d with
    variance chosen so that tokens have about unit variance."""
    rng = np.random.default_rng(seed)
    dp = 3 * patch * patch
    return (rng.standard_normal((dp, d_model)) * np.sqrt(3.0 / dp)).astype(np.float32)


def visual_embeddings(frame, patch, w_proj):
    """Visual token embeddings [N*N, d] float32 of one frame."""
    x = patch_pixels(frame, patch).astype(np.float32) / 127.5 - 1.0
    return (x @ w_proj).astype(np.float32)


def text_embeddings(n_text, d_model, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n_text, d_model)).astype(np.float32)
